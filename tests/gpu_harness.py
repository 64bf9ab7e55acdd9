"""Helpers for the GPU parity tests: run one call sequence through the C ABI
and through the oracle on the same seeded images, and compare every byte."""
import numpy as np
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V


class GpuCase:
    """Cache in HBM + engine, mirrored by host images the oracle works on."""

    def __init__(self, shape, layout, path, cache_u16, pool_u16, own_pool=True, own_streams=True,
                 **cfgkw):
        self.shape, self.layout = shape, layout
        self.cfg = B.make_config(shape, layout, path, **cfgkw)
        self.oshape = O.shape_of(shape, layout)
        self.ref_cache = cache_u16.copy()
        self.ref_pool = pool_u16.copy()
        self.dev_cache = torch.from_numpy(cache_u16.view(np.int16).copy()).cuda()
        self.pinned = None
        self.streams = None
        pool_ptr = so = si = 0
        if not own_pool:
            self.pinned = torch.empty(pool_u16.size, dtype=torch.int16).pin_memory()
            pool_ptr = self.pinned.data_ptr()
        if not own_streams:
            self.streams = (torch.cuda.Stream(), torch.cuda.Stream())
            so, si = self.streams[0].cuda_stream, self.streams[1].cuda_stream
        torch.cuda.synchronize()
        self.eng = B.Engine(self.cfg, self.dev_cache.data_ptr(), pool_ptr, so, si)
        self.pool_u8 = self.eng.host_pool_array()
        assert self.pool_u8.size == pool_u16.size * 2
        self.pool_u8[:] = pool_u16.view(np.uint8)

    def rotate(self, rot, expect=0):
        rc = self.eng.kv_rotate(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
        assert rc == expect, f"library returned {rc}, wanted {expect}"
        rco = O.rotate(self.oshape, self.ref_cache.view(np.uint8), self.ref_pool.view(np.uint8),
                       rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
        assert rco == expect, f"oracle returned {rco}, wanted {expect}"

    def swap_out(self, ids, slots, expect=0):
        assert self.eng.kv_swap_out(ids, slots) == expect
        assert O.swap_out(self.oshape, self.ref_cache.view(np.uint8), self.ref_pool.view(np.uint8),
                          ids, slots) == expect

    def swap_in(self, slots, ids, expect=0):
        assert self.eng.kv_swap_in(slots, ids) == expect
        assert O.swap_in(self.oshape, self.ref_cache.view(np.uint8), self.ref_pool.view(np.uint8),
                         slots, ids) == expect

    def wait(self):
        assert self.eng.kv_wait() == 0

    def check(self):
        """Whole cache and whole pool, byte for byte."""
        self.wait()
        got_cache = self.dev_cache.cpu().numpy().view(np.uint16)
        got_pool = self.pool_u8.view(np.uint16)
        bad_c = np.flatnonzero(got_cache != self.ref_cache)
        bad_p = np.flatnonzero(got_pool != self.ref_pool)
        assert bad_c.size == 0, f"cache differs at {bad_c.size} elements, first {bad_c[:4]}"
        assert bad_p.size == 0, f"pool differs at {bad_p.size} elements, first {bad_p[:4]}"

    def close(self):
        self.eng.kv_destroy()


def make_case(name_or_shape, layout, path, rot=None, seed=None, **kw):
    if isinstance(name_or_shape, str):
        shape = W.SHAPES[name_or_shape]
        rot = rot or W.config_rotation(name_or_shape)
        seed = W.value_seed(name_or_shape) if seed is None else seed
    else:
        shape = name_or_shape
        seed = 1234 if seed is None else seed
    cache, pool = V.make_images(shape, layout, rot, seed)
    return GpuCase(shape, layout, path, cache, pool, **kw), rot
