"""The library's block table with eager rotation against the oracle's, on the
same schedules: mappings, counters and every byte of cache and pool must agree,
and each request's tokens must be readable through the library's mapping."""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V
from tests.tablemodel import LogicalKV, DIRTY, FULL, SYNCED, HOST

pytestmark = pytest.mark.gpu

COUNT_MAP = dict(free_hbm="free_hbm_blocks", free_slots="free_host_slots", copied_eager="copied_eager",
                 copied_preempt="copied_preempt", dropped_synced="dropped_synced", swapped_in="swapped_in")


class BothSides:
    """Oracle table on host images and library table on the GPU, in lock step."""

    def __init__(self, shape, layout, max_req=8, seed=1, **cfgkw):
        self.shape, self.layout = shape, layout
        self.os = O.shape_of(shape, layout)
        self.ot = O.Table(self.os, max_req)
        self.ref_cache = np.zeros(V.n_cache_elems(shape), np.uint16)
        self.ref_pool = np.zeros(V.n_pool_elems(shape), np.uint16)
        self.model = LogicalKV(shape, layout, seed)
        self.cfg = B.make_config(shape, layout, **cfgkw)
        self.dev = torch.zeros(V.n_cache_elems(shape), dtype=torch.int16, device="cuda")
        torch.cuda.synchronize()
        self.eng = B.Engine(self.cfg, self.dev.data_ptr())
        self.pool_u8 = self.eng.host_pool_array()
        self.pool_u8[:] = 0
        self.gt = B.Table(self.eng, max_req)

    def u8(self, a):
        return a.view(np.uint8)

    def append(self, req, n):
        before = self.ot.blocks(req)
        old_len = before["len"] if before else 0
        rc_o, ids_o = self.ot.append(req, n)
        rc_g, ids_g = self.gt.kv_table_append(req, n)
        assert rc_o == rc_g and ids_o == ids_g
        if rc_o == O.OK and n > 0:
            toks = self.model.grow(req, n)
            ids = self.ot.blocks(req)["ids"]
            self.model.write_new_tokens(self.ref_cache, ids, old_len, toks)
            # the same "model writes" on the GPU, after earlier transfers have landed
            assert self.eng.kv_wait() == 0
            dv = self.dev.view(self.shape.n_layers, 2, self.shape.n_hbm_blocks, self.shape.block_size,
                               self.shape.n_kv_heads, self.shape.head_dim)
            P = self.shape.block_size
            tt = torch.from_numpy(toks.view(np.int16)).cuda()
            for k in range(n):
                tok = old_len + k
                dv[:, :, ids[tok // P], tok % P] = tt[k]
            torch.cuda.synchronize()
        elif rc_o == O.OK and before is None:
            self.model.tokens[req] = np.zeros((0,) + self.model.token_dims(), np.uint16)
        return rc_o

    def eager(self, budget):
        rc_o, n_o = self.ot.eager(self.u8(self.ref_cache), self.u8(self.ref_pool), budget)
        rc_g, n_g = self.gt.kv_table_eager(budget)
        assert (rc_o, n_o) == (rc_g, n_g)
        return n_o

    def rotate(self, pre, res):
        rc_o = self.ot.rotate(self.u8(self.ref_cache), self.u8(self.ref_pool), pre, res)
        rc_g = self.gt.kv_table_rotate(pre, res)
        assert rc_o == rc_g, (rc_o, rc_g)
        return rc_o

    def rotate_eager(self, pre, res, budget):
        rc_o, n_o = self.ot.rotate_eager(self.u8(self.ref_cache), self.u8(self.ref_pool), pre, res, budget)
        rc_g, n_g = self.gt.kv_table_rotate_eager(pre, res, budget)
        assert (rc_o, n_o) == (rc_g, n_g), (rc_o, n_o, rc_g, n_g)
        return rc_o, n_o

    def finish(self, req):
        assert self.eng.kv_wait() == 0
        rc_o, rc_g = self.ot.finish(req), self.gt.kv_table_finish(req)
        assert rc_o == rc_g
        if rc_o == O.OK:
            self.model.drop(req)
        return rc_o

    def check(self, max_req=8):
        assert self.eng.kv_wait() == 0
        got_cache = self.dev.cpu().numpy().view(np.uint16)
        got_pool = self.pool_u8.view(np.uint16)
        for r in range(max_req):
            assert self.ot.blocks(r) == self.gt.kv_table_blocks(r), f"mapping of request {r}"
        co, cg = self.ot.counts(), self.gt.kv_table_get_counts()
        assert {COUNT_MAP[k]: v for k, v in co.items()} == cg
        assert np.array_equal(got_cache, self.ref_cache), "cache differs from the oracle"
        assert np.array_equal(got_pool, self.ref_pool), "pool differs from the oracle"
        self.model.check(self.gt.kv_table_blocks, got_cache, got_pool,
                         dict(free_hbm=cg["free_hbm_blocks"], free_slots=cg["free_host_slots"]))

    def close(self):
        self.gt.kv_table_destroy()
        self.eng.kv_destroy()


@pytest.mark.parametrize("layout", [B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST])
def test_eager_rotation_lifecycle(layout):
    sh = W.KVShape(2, 2, 64, 4, n_hbm_blocks=12, n_host_slots=20)
    s = BothSides(sh, layout)
    s.append(0, 14)
    s.append(1, 14)
    assert s.eager(100) == 6
    s.check()
    c0 = s.gt.kv_table_get_counts()
    assert s.rotate([0], []) == 0
    c1 = s.gt.kv_table_get_counts()
    assert c1["copied_preempt"] - c0["copied_preempt"] == 1 and c1["dropped_synced"] - c0["dropped_synced"] == 3
    st = s.eng.kv_wait(); assert st == 0
    assert s.eng.kv_last_stats()["bytes_out"] == B.kv_block_bytes(s.cfg)     # one block crossed the link
    s.check()
    s.append(2, 9)
    assert s.rotate([1, 2], [0]) == 0          # duplex: two out, one back in
    s.check()
    s.append(0, 3)                             # the resumed tail fills up (FULL), one token starts a new block
    assert s.gt.kv_table_blocks(0)["states"] == [SYNCED, SYNCED, SYNCED, FULL, DIRTY]
    assert s.rotate([0], [1, 2]) == 0
    s.check()
    assert s.finish(1) == 0
    assert s.rotate([], [0]) == 0
    s.check()
    s.close()


def test_engine_outlives_its_table():
    sh = W.KVShape(1, 1, 64, 4, n_hbm_blocks=4, n_host_slots=4)
    s = BothSides(sh, B.KV_HOST_BLOCK_FIRST)
    s.append(0, 6)
    assert s.eng.kv_destroy() == B.KV_EBUSY          # refused: the table still points at the engine
    assert s.rotate([0], []) == 0                    # and both still work
    s.check()
    assert s.gt.kv_table_destroy() == 0
    assert s.eng.kv_destroy() == 0


def test_race_rule_on_the_gpu():
    sh = W.KVShape(1, 1, 64, 4, n_hbm_blocks=4, n_host_slots=16)
    s = BothSides(sh, B.KV_HOST_BLOCK_FIRST)
    s.append(0, 8)
    assert s.rotate([0], []) == 0
    s.append(1, 16)
    assert s.eager(10) == 4
    assert s.rotate([1], [0]) == 0             # room only through request 1's synced drops
    s.check()
    s.append(2, 8)
    assert s.rotate([0, 2], [1]) == B.KV_ENOSPC    # request 2's blocks are being copied out: not reusable
    s.check()
    assert s.eager(10) == 2
    assert s.rotate([0, 2], [1]) == 0
    s.check()
    assert s.rotate([9], []) == B.KV_EINVAL and s.rotate([1, 1], []) == B.KV_EINVAL
    assert s.rotate([], [1]) == B.KV_EINVAL
    s.check()
    s.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY])
@pytest.mark.parametrize("seed", [0, 1])
@pytest.mark.parametrize("layout", [B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST])
def test_random_schedules_match_the_oracle(layout, seed, path):
    sh = W.KVShape(2, 2, 64, 4, n_hbm_blocks=24, n_host_slots=40)
    s = BothSides(sh, layout, max_req=6, seed=seed, path=path)
    rng = np.random.default_rng(500 + seed)
    for step in range(120):
        op = rng.integers(0, 10)
        reqs = list(s.model.tokens)
        resident = [r for r in reqs if s.ot.blocks(r)["resident"]]
        rotary = [r for r in reqs if not s.ot.blocks(r)["resident"]]
        if op <= 3:
            cand = resident + [r for r in range(6) if r not in reqs]
            if cand:
                s.append(int(rng.choice(cand)), int(rng.integers(0, 11)))
        elif op <= 5:
            s.eager(int(rng.integers(0, 5)))
        elif op <= 8:
            pre, res = [r for r in resident if rng.random() < 0.4], [r for r in rotary if rng.random() < 0.5]
            if rng.random() < 0.5:
                s.rotate(pre, res)
            else:
                s.rotate_eager(pre, res, int(rng.integers(0, 6)))
        elif reqs:
            s.finish(int(rng.choice(reqs)))
        if step % 10 == 9:
            s.check(6)
    s.check(6)
    c = s.gt.kv_table_get_counts()
    assert c["copied_eager"] > 0 and c["copied_preempt"] > 0 and c["dropped_synced"] > 0 and c["swapped_in"] > 0
    s.close()


def test_llama_shape_preemption_moves_one_block_per_request():
    """Llama-3-8B block shape: 16 requests of 1000 tokens, eagerly synced while
    they run; preempting 8 and resuming 8 others moves 8 dirty tails out, not 8 x 63 blocks."""
    sh = W.KVShape(32, 8, 128, 16, n_hbm_blocks=1100, n_host_slots=1100)
    os_ = O.shape_of(sh, 0)
    dev = torch.empty(V.n_cache_elems(sh), dtype=torch.int16, device="cuda").random_()
    torch.cuda.synchronize()
    eng = B.Engine(B.make_config(sh), dev.data_ptr())
    tab = B.Table(eng, 32)
    blk = B.kv_block_bytes(eng.cfg)
    for r in range(16):
        assert tab.kv_table_append(r, 1000)[0] == 0          # 62 full blocks + a tail of 8 tokens
    rc, n = tab.kv_table_eager(10 ** 6)
    assert (rc, n) == (0, 16 * 62)
    assert eng.kv_wait() == 0
    assert eng.kv_last_stats()["bytes_out"] == 16 * 62 * blk
    assert tab.kv_table_rotate(list(range(8)), []) == 0
    assert eng.kv_wait() == 0
    assert eng.kv_last_stats()["bytes_out"] == 8 * blk       # the dirty tails only
    # contents of a preempted request are in its slots: compare with what HBM held (blocks were random)
    assert tab.kv_table_rotate(list(range(8, 16)), list(range(8))) == 0
    assert eng.kv_wait() == 0
    st = eng.kv_last_stats()
    assert st["bytes_out"] == 8 * blk and st["bytes_in"] == 8 * 63 * blk and st["path_used"] == B.KV_PATH_FUSED
    c = tab.kv_table_get_counts()
    assert c["copied_preempt"] == 16 and c["dropped_synced"] == 16 * 62 and c["swapped_in"] == 8 * 63
    # every resumed block equals its DRAM copy (state SYNCED means exactly that)
    pool = eng.host_pool_array().view(np.uint16)
    pv = pool.reshape((sh.n_host_slots,) + sh.block_dims())
    dv = dev.view(sh.n_layers, 2, sh.n_hbm_blocks, sh.block_size, sh.n_kv_heads, sh.head_dim)
    for r in range(8):
        b = tab.kv_table_blocks(r)
        assert b["resident"] and b["states"] == [SYNCED] * 63
        got = dv[:, :, torch.tensor(b["ids"], device="cuda")].cpu().numpy().view(np.uint16)   # [L,2,n,P,H,D]
        assert np.array_equal(got.transpose(2, 0, 1, 3, 4, 5), pv[b["slots"]])
    tab.kv_table_destroy()
    eng.kv_destroy()


@pytest.mark.parametrize("path,chunk_layers", [(B.KV_PATH_AUTO, 0), (B.KV_PATH_ZEROCOPY, 0), (B.KV_PATH_AUTO, 3)])
def test_back_to_back_table_calls_without_waiting(path, chunk_layers):
    """Eager copies, preemptions and resumptions enqueued back to back: blocks that
    one call vacates are refilled by the next while the first may still be running,
    so this only passes if the table orders its transfers across the two streams
    (on the two-kernel path every rotation puts one kernel on each stream; with
    chunk_layers every transfer is several launches, layer by layer)."""
    sh = W.KVShape(8, 8, 128, 16, n_hbm_blocks=96, n_host_slots=256)     # 512 KiB blocks
    s = BothSides(sh, B.KV_HOST_BLOCK_FIRST, max_req=6, seed=7, path=path, chunk_layers=chunk_layers)
    for r in range(4):
        s.append(r, 16 * 22 + 5)              # 22 full blocks + a tail; 4 x 23 = 92 of 96 blocks
    s.check(6)
    for rep in range(3):
        s.eager(1000)                         # out-only on stream_out
        s.rotate([0, 1], [])                  # tails out, synced blocks dropped
        s.rotate([], [0])                     # in-only on stream_in, into blocks just vacated
        s.rotate([2], [1])                    # fused
        s.rotate([3, 0], [2])                 # fused, reusing what the previous call released
        s.rotate([], [3])
        s.rotate([1], [0])
        s.rotate([], [1])
        # all four are resident again; nothing was waited for in between
    s.check(6)
    s.close()


def test_eager_copies_ride_in_the_rotation_transfer():
    """Llama shape: two requests leave (synced but for their tails), two come back, and
    the eager step of a third, which stays, goes out in the same launch."""
    sh = W.KVShape(32, 8, 128, 16, n_hbm_blocks=512, n_host_slots=512)
    s = BothSides(sh, B.KV_HOST_BLOCK_FIRST, max_req=8)
    P = sh.block_size
    for r in (0, 1, 2, 3):
        assert s.append(r, 20 * P + 3) == 0           # 20 full blocks and a tail each
    assert s.eager(200) == 80
    assert s.rotate([2, 3], []) == 0                  # 2 and 3 wait in DRAM
    assert s.append(4, 40 * P + 5) == 0               # 40 full blocks, never synced
    s.check()
    rc, n = s.rotate_eager([0, 1], [2, 3], 30)
    assert (rc, n) == (0, 30)
    s.check()
    st = s.eng.kv_last_stats()
    assert st["n_launches"] == 1                      # one transfer: 2 tails + 30 eager out, 42 in
    blk = B.kv_block_bytes(s.cfg)
    assert st["bytes_out"] == 32 * blk and st["bytes_in"] == 42 * blk
    assert s.gt.kv_table_blocks(4)["states"][:31] == [O.SYNCED] * 30 + [O.FULL]
    s.close()


def test_finish_waits_only_for_transfers_on_its_own_blocks():
    """An eager copy of ~0.5 GiB is in flight (request 0's 256 full blocks).  Finishing
    request 2, none of whose blocks the copy names, returns while it still runs;
    finishing request 0 returns only when it is done."""
    sh = W.KVShape(32, 8, 128, 16, n_hbm_blocks=400, n_host_slots=400)     # 2 MiB blocks
    dev = torch.empty(V.n_cache_elems(sh), dtype=torch.int16, device="cuda").random_()
    torch.cuda.synchronize()
    eng = B.Engine(B.make_config(sh), dev.data_ptr())
    tab = B.Table(eng, 4)
    P = sh.block_size
    assert tab.kv_table_append(0, 256 * P)[0] == 0
    assert tab.kv_table_append(1, 2 * P)[0] == 0
    assert tab.kv_table_append(2, P // 2)[0] == 0            # a partly filled block: nothing to copy
    assert tab.kv_table_eager(256) == (0, 256)               # request 0 only
    assert eng.kv_query() == B.KV_EBUSY, "the copy was done before the call returned"
    assert tab.kv_table_finish(2) == 0
    assert eng.kv_query() == B.KV_EBUSY, "finishing an uninvolved request waited for the copy"
    assert tab.kv_table_finish(0) == 0
    assert eng.kv_query() == 0, "request 0's blocks were freed while their copy still ran"
    # the copies are what the cache held
    got = tab.kv_table_blocks(1)
    assert got["len"] == 2 * P
    assert eng.kv_wait() == 0
    assert eng.kv_last_stats()["bytes_out"] == 256 * (2 << 20)
    assert tab.kv_table_eager(10) == (0, 2)                  # request 1, afterwards
    assert tab.kv_table_finish(1) == 0                       # its copy may be in flight: waits
    assert eng.kv_query() == 0
    assert tab.kv_table_get_counts()["free_hbm_blocks"] == 400
    tab.kv_table_destroy()
    eng.kv_destroy()
