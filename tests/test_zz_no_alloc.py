"""kv_rotate_static, the entry point that allocates nothing, against kv_rotate:
the same calls on the same images must leave the same bytes in cache and pool
(and both must equal the oracle's), on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V
from tests.gpu_harness import make_case

pytestmark = pytest.mark.gpu


class StaticSide:
    """Cache in HBM and a pinned pool of the caller's, no engine."""

    def __init__(self, shape, layout, cache_u16, pool_u16, **cfgkw):
        self.cfg = B.make_config(shape, layout, **cfgkw)
        self.dev = torch.from_numpy(cache_u16.view(np.int16).copy()).cuda()
        self.pinned = torch.from_numpy(pool_u16.view(np.int16).copy()).pin_memory()
        self.stream = torch.cuda.Stream()
        torch.cuda.synchronize()

    def rotate(self, rot, expect=0):
        rc = B.kv_rotate_static(self.cfg, self.dev.data_ptr(), self.pinned.data_ptr(), self.stream.cuda_stream,
                                rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
        assert rc == expect, f"kv_rotate_static returned {rc}, wanted {expect}"

    def images(self):
        self.stream.synchronize()
        return self.dev.cpu().numpy().view(np.uint16), self.pinned.numpy().view(np.uint16)


def second_rotation(shape, first, n_out, n_in, seed):
    """A smaller rotation over blocks and slots the first one did not name."""
    rng = np.random.default_rng(seed)
    free_b = np.setdiff1d(np.arange(shape.n_hbm_blocks), np.concatenate([first.out_ids, first.in_ids]))
    free_s = np.setdiff1d(np.arange(shape.n_host_slots), np.concatenate([first.out_slots, first.in_slots]))
    b = rng.permutation(free_b)[:n_out + n_in].astype(np.int32)
    s = rng.permutation(free_s)[:n_out + n_in].astype(np.int32)
    return W.Rotation(b[:n_out], s[:n_out], b[n_out:], s[n_out:])


@pytest.mark.parametrize("name,layout", [("small8b", B.KV_HOST_BLOCK_FIRST), ("small8b", B.KV_HOST_LAYER_FIRST),
                                         ("ragged", B.KV_HOST_BLOCK_FIRST), ("tiny", B.KV_HOST_BLOCK_FIRST)])
def test_two_calls_in_a_row_match_kv_rotate(name, layout):
    case, rot = make_case(name, layout, B.KV_PATH_AUTO)
    shape = case.shape
    cache0, pool0 = case.ref_cache.copy(), case.ref_pool.copy()
    st = StaticSide(shape, layout, cache0, pool0)
    small = second_rotation(shape, rot, 3, 2, seed=11)
    # the existing entry point: two calls, the second smaller, no wait between them
    case.rotate(rot)
    case.rotate(small)
    case.check()                                    # engine == oracle
    want_cache = case.dev_cache.cpu().numpy().view(np.uint16)
    want_pool = case.pool_u8.view(np.uint16).copy()
    # the same two calls through the entry point that allocates nothing
    st.rotate(rot)
    st.rotate(small)
    got_cache, got_pool = st.images()
    assert np.array_equal(got_cache, want_cache), "cache differs from kv_rotate's"
    assert np.array_equal(got_pool, want_pool), "pool differs from kv_rotate's"
    # and back: the inverse of the small one, then of the large one, then a single direction each
    for r in (small.inverse(), rot.inverse(),
              W.Rotation(rot.out_ids[:4], rot.out_slots[:4], rot.in_ids[:0], rot.in_slots[:0]),
              W.Rotation(rot.out_ids[:0], rot.out_slots[:0], rot.in_ids[:3], rot.in_slots[:3])):
        case.rotate(r)
        st.rotate(r)
    case.check()
    got_cache, got_pool = st.images()
    assert np.array_equal(got_cache, case.dev_cache.cpu().numpy().view(np.uint16))
    assert np.array_equal(got_pool, case.pool_u8.view(np.uint16))
    case.close()


def test_in_heavy_and_out_heavy_lists_match_kv_rotate():
    """Llama-3-8B block shape: the in list three times the out list (out tiles
    spread over the in tiles), then the reverse."""
    shape = W.KVShape(32, 8, 128, 16, n_hbm_blocks=160, n_host_slots=160)
    rot = W.simple_rotation(shape, 12, 36, seed=5)
    case, _ = make_case(shape, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO, rot=rot)
    st = StaticSide(shape, B.KV_HOST_BLOCK_FIRST, case.ref_cache.copy(), case.ref_pool.copy())
    for r in (rot, rot.inverse()):
        case.rotate(r)
        st.rotate(r)
        case.check()
        got_cache, got_pool = st.images()
        assert np.array_equal(got_cache, case.dev_cache.cpu().numpy().view(np.uint16))
        assert np.array_equal(got_pool, case.pool_u8.view(np.uint16))
    case.close()


def test_admission_and_the_size_limit():
    case, rot = make_case("tiny", B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO)
    shape = case.shape
    st = StaticSide(shape, B.KV_HOST_BLOCK_FIRST, case.ref_cache.copy(), case.ref_pool.copy())
    before = st.images()
    bad = [
        (W.Rotation(np.array([0, 0], np.int32), np.array([1, 2], np.int32), rot.in_ids[:0], rot.in_slots[:0]), B.KV_EDUP),
        (W.Rotation(np.array([shape.n_hbm_blocks], np.int32), np.array([1], np.int32), rot.in_ids[:0], rot.in_slots[:0]),
         B.KV_ERANGE),
        (W.Rotation(np.array([3], np.int32), np.array([1], np.int32), np.array([3], np.int32), np.array([2], np.int32)),
         B.KV_EOVERLAP),
        (W.Rotation(np.array([3], np.int32), np.array([1], np.int32), np.array([4], np.int32), np.array([1], np.int32)),
         B.KV_EOVERLAP),
    ]
    for r, code in bad:
        st.rotate(r, expect=code)
        assert O.validate(case.oshape, r.out_ids, r.out_slots, r.in_ids, r.in_slots) == code
    after = st.images()
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    # beyond the scratch array: refused before anything else is looked at
    big = W.KVShape(1, 1, 8, 1, n_hbm_blocks=2 * B.KV_STATIC_MAX_BLOCKS, n_host_slots=2 * B.KV_STATIC_MAX_BLOCKS)
    n = B.KV_STATIC_MAX_BLOCKS // 2 + 1
    ids = np.arange(2 * n, dtype=np.int32)
    cfg = B.make_config(big)
    dev = torch.zeros(B.kv_cache_bytes(cfg), dtype=torch.uint8, device="cuda")
    pin = torch.zeros(B.kv_pool_bytes(cfg), dtype=torch.uint8).pin_memory()
    rc = B.kv_rotate_static(cfg, dev.data_ptr(), pin.data_ptr(), 0, ids[:n], ids[:n], ids[n:], ids[n:])
    assert rc == B.KV_E2BIG
    # the largest admissible call: every id list travels through several launches
    n = B.KV_STATIC_MAX_BLOCKS // 2
    dev.random_()
    want = dev.cpu().numpy().copy()
    rc = B.kv_rotate_static(cfg, dev.data_ptr(), pin.data_ptr(), 0, ids[:n], ids[:n], ids[n:2 * n], ids[n:2 * n])
    assert rc == 0
    torch.cuda.synchronize()
    sh_o = O.shape_of(big, 0)
    ref_pool = np.zeros(B.kv_pool_bytes(cfg), np.uint8)
    assert O.rotate(sh_o, want, ref_pool, ids[:n], ids[:n], ids[n:2 * n], ids[n:2 * n]) == 0
    assert np.array_equal(dev.cpu().numpy(), want) and np.array_equal(pin.numpy(), ref_pool)
    # a wrong path, a pointer that is no device allocation
    cfg2 = B.make_config(shape, path=B.KV_PATH_SDMA_STAGED)
    assert B.kv_rotate_static(cfg2, st.dev.data_ptr(), st.pinned.data_ptr(), 0, rot.out_ids, rot.out_slots,
                              rot.in_ids, rot.in_slots) == B.KV_EUNSUP
    host = np.zeros(B.kv_cache_bytes(st.cfg), np.uint8)
    assert B.kv_rotate_static(st.cfg, host.ctypes.data, st.pinned.data_ptr(), 0, rot.out_ids, rot.out_slots,
                              rot.in_ids, rot.in_slots) == B.KV_EINVAL
    case.close()


def test_llama3_8b_full_size_matches_kv_rotate():
    """configs[1] in bench.py's shape: 16 GiB cache, 128 scattered blocks each way."""
    shape = W.SHAPES["llama3_8b"]
    rot = W.config_rotation("llama3_8b")
    seed = W.value_seed("llama3_8b")
    cfg = B.make_config(shape)
    caches = [W.cache_image(shape, seed, device="cuda") for _ in range(2)]
    assert torch.equal(caches[0].view(torch.int16), caches[1].view(torch.int16))
    eng = B.Engine(cfg, caches[0].data_ptr())
    pool_a = eng.host_pool_array()
    pinned = torch.empty(B.kv_pool_bytes(cfg), dtype=torch.uint8).pin_memory()
    pool_b = pinned.numpy()
    staged = W.staged_blocks(shape, len(rot.in_slots), seed + 50, device="cuda").view(torch.int16).cpu().numpy()
    for pool in (pool_a, pool_b):
        pool[:] = 0x5A
        pool.view(np.int16).reshape((shape.n_host_slots,) + shape.block_dims())[rot.in_slots] = staged
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    for r in (rot, rot.inverse(), rot):
        assert eng.kv_rotate(r.out_ids, r.out_slots, r.in_ids, r.in_slots) == 0
        assert B.kv_rotate_static(cfg, caches[1].data_ptr(), pinned.data_ptr(), stream.cuda_stream,
                                  r.out_ids, r.out_slots, r.in_ids, r.in_slots) == 0
    assert eng.kv_wait() == 0
    stream.synchronize()
    assert torch.equal(caches[0].view(torch.int16), caches[1].view(torch.int16)), "cache differs from kv_rotate's"
    assert np.array_equal(pool_a, pool_b), "pool differs from kv_rotate's"
    # and the rotation really happened: the swapped-in blocks hold the staged bytes
    got = caches[1].view(torch.int16)[:, :, torch.from_numpy(rot.in_ids).long().cuda()].cpu().numpy()
    assert np.array_equal(got.transpose(2, 0, 1, 3, 4, 5), staged)
    eng.kv_destroy()


def test_replays_of_a_captured_call():
    """The call for which the entry point exists: recorded into a HIP graph and
    replayed.  Between replays the program changes what the blocks and slots hold,
    with its own eager work and synchronisations, and every replay must move the
    bytes that are there at that moment."""
    case, rot = make_case("small8b", B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO)
    shape, cfg = case.shape, case.cfg
    dev = torch.from_numpy(case.ref_cache.view(np.int16).copy()).cuda()
    pinned = torch.from_numpy(case.ref_pool.view(np.int16).copy()).pin_memory()
    stream = torch.cuda.Stream()
    args = (rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
    # first call outside any capture: it looks up the scratch array's address on this device
    assert B.kv_rotate_static(cfg, dev.data_ptr(), pinned.data_ptr(), stream.cuda_stream, *args) == 0
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        rc = B.kv_rotate_static(cfg, dev.data_ptr(), pinned.data_ptr(), torch.cuda.current_stream().cuda_stream, *args)
    assert rc == 0
    dv = dev.view(shape.n_layers, 2, shape.n_hbm_blocks, shape.block_size, shape.n_kv_heads, shape.head_dim)
    pv = pinned.view((shape.n_host_slots,) + shape.block_dims())
    out_ids, in_ids = torch.from_numpy(rot.out_ids).long().cuda(), torch.from_numpy(rot.in_ids).long().cuda()
    g = torch.Generator(device="cuda").manual_seed(5)
    for k in range(4):
        # new contents for the blocks that leave and for the slots that come in
        fresh = torch.randint(-32768, 32767, dv[:, :, out_ids].shape, generator=g, dtype=torch.int16, device="cuda")
        dv[:, :, out_ids] = fresh
        incoming = torch.from_numpy(np.random.default_rng(k).integers(-32768, 32767, size=(len(rot.in_slots),) +
                                    shape.block_dims(), dtype=np.int16))
        pv[torch.from_numpy(rot.in_slots).long()] = incoming
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(pv[torch.from_numpy(rot.out_slots).long()], fresh.cpu().permute(2, 0, 1, 3, 4, 5)), f"replay {k}: out"
        assert torch.equal(dv[:, :, in_ids].cpu().permute(2, 0, 1, 3, 4, 5), incoming), f"replay {k}: in"
    case.close()


@pytest.mark.parametrize("seed", range(4))
def test_random_cases_match_the_oracle(seed):
    """Random small shapes, layouts and launch knobs through kv_rotate_static, two or
    three calls each on one stream without a wait in between, against the oracle."""
    rng = np.random.default_rng(8100 + seed)
    for k in range(40):
        sh = W.KVShape(int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.choice([4, 8, 20, 40, 64])),
                       int(rng.integers(1, 8)), n_hbm_blocks=int(rng.integers(6, 40)), n_host_slots=int(rng.integers(6, 40)))
        layout = int(rng.choice([B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST]))
        hbm_layout = int(rng.choice([B.KV_HBM_LAYER_FIRST, B.KV_HBM_BLOCK_FIRST]))
        kw = dict(hbm_layout=hbm_layout)
        if rng.random() < 0.4:
            kw["vecs_per_lane"] = int(rng.choice([1, 2, 4, 8]))
        if rng.random() < 0.4:
            kw["max_copy_wgs"] = int(rng.choice([1, 3, 40]))
        n16 = lambda nb: sh.n_layers * 2 * nb * sh.block_size * sh.n_kv_heads * sh.head_dim
        cache = rng.integers(0, 65536, n16(sh.n_hbm_blocks), dtype=np.uint16)
        pool = rng.integers(0, 65536, n16(sh.n_host_slots), dtype=np.uint16)
        st = StaticSide(sh, layout, cache, pool, **kw)
        oshape = O.shape_of(sh, layout, hbm_layout)
        for step in range(int(rng.integers(2, 4))):
            cap = min(sh.n_hbm_blocks, sh.n_host_slots)
            n_out = int(rng.integers(0, cap // 2 + 1))
            n_in = int(rng.integers(0, cap - n_out - cap // 4 + 1))
            ids = rng.permutation(sh.n_hbm_blocks)[:n_out + n_in].astype(np.int32)
            slots = rng.permutation(sh.n_host_slots)[:n_out + n_in].astype(np.int32)
            rot = W.Rotation(ids[:n_out], slots[:n_out], ids[n_out:], slots[n_out:])
            st.rotate(rot)
            assert O.rotate(oshape, cache.view(np.uint8), pool.view(np.uint8), rot.out_ids, rot.out_slots,
                            rot.in_ids, rot.in_slots) == 0
        got_cache, got_pool = st.images()
        what = f"seed {seed} case {k}: {sh}, layout {layout}, {kw}"
        assert np.array_equal(got_cache, cache), what + ": cache"
        assert np.array_equal(got_pool, pool), what + ": pool"
