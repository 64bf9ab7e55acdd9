"""Helpers for the GPU parity tests: run one call sequence through the C ABI
and through the oracle on the same seeded images, and compare every byte."""
from concurrent.futures import ThreadPoolExecutor

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
        self.oshape = O.shape_of(shape, layout, cfgkw.get("hbm_layout", 0))
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
    cache, pool = V.make_images(shape, layout, rot, seed, hbm_layout=kw.get("hbm_layout", 0))
    return GpuCase(shape, layout, path, cache, pool, **kw), rot


_WORKERS = 8
_pool = ThreadPoolExecutor(_WORKERS)


def _over(n, fn):
    """fn(a, b) on slices [a, b) that tile range(n), on the worker threads (NumPy
    copies and comparisons of large arrays release the interpreter lock);
    returns the results in order."""
    step = -(-n // _WORKERS)
    return list(_pool.map(lambda a: fn(a, min(n, a + step)), range(0, n, step)))


class BigCase:
    """Full-size check that needs little host memory.

    The cache is drawn on the GPU.  The oracle works on host images that are
    allocated lazily: only the blocks and slots a rotation (or a reader) names
    are ever filled (with the exact bytes the GPU holds) or touched, which is
    all the oracle reads or writes.  Named blocks and slots are compared with
    the oracle's result byte for byte; every other block is compared with a
    regenerated image on the GPU, every other slot with the fill pattern it was
    given.  Device <-> host traffic of the check itself goes in pieces of about
    1 GiB; `say` (a callable taking one string) reports progress.
    """

    FILL = 0xA5
    PIECE = 1 << 30

    def __init__(self, name, layout=B.KV_HOST_BLOCK_FIRST, path=B.KV_PATH_AUTO, shape=None, say=None, **cfgkw):
        self.name, self.layout = name, layout
        self.say = say or (lambda msg: None)
        self.shape = shape or W.SHAPES[name]
        self.seed = W.value_seed(name)
        self.cfg = B.make_config(self.shape, layout, path, **cfgkw)
        self.oshape = O.shape_of(self.shape, layout)
        self.per_piece = max(1, self.PIECE // O.block_bytes(self.oshape))
        self.cache = W.cache_image(self.shape, self.seed, device="cuda")
        torch.cuda.synchronize()
        self.say(f"{name}: cache of {O.cache_bytes(self.oshape) >> 30} GiB drawn")
        self.eng = B.Engine(self.cfg, self.cache.data_ptr())
        self.pool_u8 = self.eng.host_pool_array()
        _over(self.pool_u8.size, lambda a, b: self.pool_u8[a:b].fill(self.FILL))
        self.say(f"{name}: pool of {O.pool_bytes(self.oshape) >> 30} GiB filled")
        self.ref_cache = np.empty(O.cache_bytes(self.oshape), dtype=np.uint8)   # lazily backed
        self.ref_pool = np.empty(O.pool_bytes(self.oshape), dtype=np.uint8)
        self.touched_blocks, self.touched_slots = set(), set()
        self._pinned = None

    # views [L,2,N,P,H,D] (uint16) of the host images and the pinned pool
    def _cv(self):
        return V.hbm_view(self.shape, self.ref_cache.view(np.uint16))

    def _pv(self, buf):
        return V.pool_view(self.shape, buf.view(np.uint16), self.layout)

    def _pieces(self, items):
        items = list(items)
        for c0 in range(0, len(items), self.per_piece):
            yield items[c0:c0 + self.per_piece]

    def _device_blocks(self, ids):
        """[L,2,len(ids),P,H,D] uint16 copy of the named blocks as the GPU holds them,
        in a pinned buffer that the next call overwrites."""
        idx = torch.tensor(ids, device="cuda")
        got = self.cache.view(torch.int16)[:, :, idx]
        if self._pinned is None:
            self._pinned = torch.empty(self.per_piece * O.block_bytes(self.oshape) // 2, dtype=torch.int16,
                                       pin_memory=True)
        host = self._pinned[:got.numel()].view(got.shape)
        host.copy_(got)
        torch.cuda.synchronize()
        return host.numpy().view(np.uint16)

    def stage(self, slots, seed_offset=50):
        """Put seeded blocks into host slots (pinned pool and reference alike)."""
        slots = np.asarray(slots)
        k = 0
        for part in self._pieces(slots):
            blocks = W.staged_blocks(self.shape, len(part), self.seed + seed_offset + k, device="cuda")
            arr = blocks.view(torch.int16).cpu().numpy().view(np.uint16).transpose(1, 2, 0, 3, 4, 5)
            pv, rv = self._pv(self.pool_u8), self._pv(self.ref_pool)

            def put(a, b):      # layers [a, b)
                pv[a:b, :, part] = arr[a:b]
                rv[a:b, :, part] = arr[a:b]
            _over(self.shape.n_layers, put)
            k += 1
        self.touched_slots.update(int(s) for s in slots)
        self.say(f"{self.name}: {len(slots)} slots staged")

    def sync_ref(self, ids, slots=(), read_only=False):
        """Bring blocks / slots that are about to be named into the reference.
        Blocks that are only read (the reader's) are mirrored for the oracle but
        stay among the blocks check() compares with the regenerated image."""
        new_b = [int(b) for b in ids if int(b) not in self.touched_blocks]
        for part in self._pieces(new_b):
            dev, cv = self._device_blocks(part), self._cv()

            def put(a, b):
                cv[a:b, :, part] = dev[a:b]
            _over(self.shape.n_layers, put)
        if not read_only:
            self.touched_blocks.update(new_b)
        new_s = [int(s) for s in slots if int(s) not in self.touched_slots]
        for part in self._pieces(new_s):
            pv, rv = self._pv(self.pool_u8), self._pv(self.ref_pool)

            def put(a, b):
                rv[a:b, :, part] = pv[a:b, :, part]
            _over(self.shape.n_layers, put)
        self.touched_slots.update(new_s)
        if new_b or new_s:
            self.say(f"{self.name}: {len(new_b)} blocks and {len(new_s)} slots mirrored on the host")

    def rotate(self, rot):
        self.sync_ref(np.concatenate([rot.out_ids, rot.in_ids]), np.concatenate([rot.out_slots, rot.in_slots]))
        assert self.eng.kv_rotate(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots) == 0
        assert O.rotate(self.oshape, self.ref_cache, self.ref_pool, rot.out_ids, rot.out_slots,
                        rot.in_ids, rot.in_slots, threads=8) == 0

    def check(self):
        assert self.eng.kv_wait() == 0
        tb = sorted(self.touched_blocks)
        ts = sorted(self.touched_slots)
        # named blocks and slots: against the oracle
        L = self.shape.n_layers
        for ids in self._pieces(tb):
            dev, cv = self._device_blocks(ids), self._cv()
            assert all(_over(L, lambda a, b: np.array_equal(dev[a:b], cv[a:b, :, ids]))), \
                "named HBM blocks differ from the oracle"
        self.say(f"{self.name}: {len(tb)} named blocks equal the oracle's")
        for sl in self._pieces(ts):
            pv, rv = self._pv(self.pool_u8), self._pv(self.ref_pool)
            assert all(_over(L, lambda a, b: np.array_equal(pv[a:b, :, sl], rv[a:b, :, sl]))), \
                "named host slots differ from the oracle"
        self.say(f"{self.name}: {len(ts)} named slots equal the oracle's")
        # every other block: against a regenerated image
        again = W.cache_image(self.shape, self.seed, device="cuda")
        for ids in self._pieces(tb):
            idx = torch.tensor(ids, device="cuda")
            again[:, :, idx] = self.cache[:, :, idx]
        assert torch.equal(again.view(torch.int16), self.cache.view(torch.int16)), "an un-named block changed"
        del again
        # every other slot: still the fill pattern
        mask = np.ones(self.shape.n_host_slots, dtype=bool)
        mask[ts] = False
        pv = self._pv(self.pool_u8)
        pat = np.uint16(self.FILL * 0x0101)
        for sl in self._pieces(np.flatnonzero(mask)):
            assert all(_over(L, lambda a, b: bool((pv[a:b, :, sl] == pat).all()))), "an un-named slot changed"
        self.say(f"{self.name}: every other block and slot unchanged")

    def close(self):
        self.eng.kv_destroy()
        del self.cache
        self._pinned = None
        torch.cuda.empty_cache()
