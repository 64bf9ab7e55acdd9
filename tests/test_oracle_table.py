"""Pins for the oracle's block table with eager rotation (paper Section 4.3.2):
logical contents tracked by a model that moves no bytes, the paper's claims
about what a preemption has to copy, the race rule, and a hand-worked case."""
import numpy as np
import pytest

from oracle import kv_oracle as O
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V
from tests.tablemodel import LogicalKV, DIRTY, FULL, SYNCED, HOST

LAYOUTS = [O.BLOCK_FIRST, O.LAYER_FIRST]
SMALL = W.KVShape(2, 2, 8, 4, n_hbm_blocks=12, n_host_slots=20)   # 4-token blocks


class OracleSide:
    """Oracle table + its images + the byte-free model, driven together."""

    def __init__(self, shape, layout, max_req=8, seed=1):
        self.shape, self.layout = shape, layout
        self.s = O.shape_of(shape, layout)
        self.t = O.Table(self.s, max_req)
        self.cache = np.zeros(V.n_cache_elems(shape), np.uint16)
        self.pool = np.zeros(V.n_pool_elems(shape), np.uint16)
        self.model = LogicalKV(shape, layout, seed)

    def u8(self, a):
        return a.view(np.uint8)

    def append(self, req, n, expect=O.OK):
        before = self.t.blocks(req)
        old_len = before["len"] if before else 0
        rc, new_ids = self.t.append(req, n)
        assert rc == expect
        if rc == O.OK:
            toks = self.model.grow(req, n)
            self.model.write_new_tokens(self.cache, self.t.blocks(req)["ids"], old_len, toks)
        return new_ids

    def eager(self, budget):
        rc, n = self.t.eager(self.u8(self.cache), self.u8(self.pool), budget)
        assert rc == O.OK
        return n

    def rotate(self, pre, res, expect=O.OK):
        assert self.t.rotate(self.u8(self.cache), self.u8(self.pool), pre, res) == expect

    def finish(self, req, expect=O.OK):
        assert self.t.finish(req) == expect
        if expect == O.OK:
            self.model.drop(req)

    def check(self):
        self.model.check(self.t.blocks, self.cache, self.pool, self.t.counts())


@pytest.mark.parametrize("layout", LAYOUTS)
def test_preemption_copies_only_what_has_no_dram_copy(layout):
    """Section 4.3.2: after eager rotation only the last dirty block needs swap-out;
    synced blocks are discarded.  Without eager rotation every block is copied."""
    o = OracleSide(SMALL, layout)
    o.append(0, 14)            # 3 full blocks + a tail of 2 tokens
    o.append(1, 14)
    assert o.t.blocks(0)["states"] == [FULL, FULL, FULL, DIRTY]
    assert o.eager(100) == 6   # the six full blocks of both requests
    assert o.t.blocks(0)["states"] == [SYNCED, SYNCED, SYNCED, DIRTY]
    o.check()
    c0 = o.t.counts()
    o.rotate([0], [])
    c1 = o.t.counts()
    assert c1["copied_preempt"] - c0["copied_preempt"] == 1      # only the dirty tail
    assert c1["dropped_synced"] - c0["dropped_synced"] == 3
    assert o.t.blocks(0)["states"] == [HOST] * 4 and not o.t.blocks(0)["resident"]
    o.check()
    # a request that was never synced pays for every block
    o2 = OracleSide(SMALL, layout)
    o2.append(0, 14)
    o2.rotate([0], [])
    assert o2.t.counts()["copied_preempt"] == 4 and o2.t.counts()["dropped_synced"] == 0
    o2.check()
    # a request whose length is a whole number of blocks and fully synced moves nothing
    o3 = OracleSide(SMALL, layout)
    o3.append(0, 8)
    assert o3.eager(10) == 2
    before = (o3.cache.copy(), o3.pool.copy())
    o3.rotate([0], [])
    assert o3.t.counts()["copied_preempt"] == 0
    assert np.array_equal(before[0], o3.cache) and np.array_equal(before[1], o3.pool)
    o3.check()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_resume_keeps_dram_copies(layout):
    o = OracleSide(SMALL, layout)
    o.append(0, 10)
    o.rotate([0], [])                       # 3 blocks copied (nothing was synced)
    o.rotate([], [0])                       # back in: all three SYNCED, tail included
    assert o.t.blocks(0)["states"] == [SYNCED] * 3 and o.t.blocks(0)["resident"]
    o.check()
    c = o.t.counts()
    o.rotate([0], [])                       # out again with no new tokens: nothing to copy
    assert o.t.counts()["copied_preempt"] == c["copied_preempt"]
    o.rotate([], [0])
    o.append(0, 1)                          # one token into the partly filled tail: dirty again
    assert o.t.blocks(0)["states"] == [SYNCED, SYNCED, DIRTY]
    o.append(0, 1)                          # fills it: 12 tokens = 3 full blocks
    assert o.t.blocks(0)["states"] == [SYNCED, SYNCED, FULL]
    slot_before = o.t.blocks(0)["slots"][2]
    assert o.eager(5) == 1
    assert o.t.blocks(0)["slots"][2] == slot_before      # its old slot is reused
    o.check()


def test_race_rule_dropped_blocks_are_reusable_copied_out_blocks_are_not():
    """Swap-in destinations may be blocks that synced drops just released, never
    blocks that the same rotation is still copying out."""
    sh = W.KVShape(1, 1, 8, 4, n_hbm_blocks=4, n_host_slots=16)
    o = OracleSide(sh, O.BLOCK_FIRST)
    o.append(0, 8)          # request 0: blocks 0, 1 (full)
    o.rotate([0], [])       # request 0 is rotary; HBM empty again
    o.append(1, 16)         # request 1 takes all four blocks
    assert o.eager(10) == 4
    # room for request 0 (2 blocks) exists only through request 1's synced drops: allowed
    o.rotate([1], [0])
    assert o.t.blocks(0)["ids"] == [0, 1] and o.t.blocks(0)["resident"]
    o.check()
    # now the other way round without syncing: request 0 holds 2, request 2 takes the other 2
    o.append(2, 8)
    assert o.t.counts()["free_hbm"] == 0
    # request 1 (4 blocks, rotary) cannot come in while 0 and 2 (unsynced) are being copied out
    c_before, p_before = o.cache.copy(), o.pool.copy()
    st0 = o.t.blocks(0)["states"]
    o.append(0, 0)
    # request 0 came back SYNCED, request 2 is FULL (never synced): only 0's two blocks can be dropped
    assert st0 == [SYNCED, SYNCED] and o.t.blocks(2)["states"] == [FULL, FULL]
    o.rotate([0, 2], [1], expect=O.ENOSPC)
    assert np.array_equal(c_before, o.cache) and np.array_equal(p_before, o.pool)
    assert o.t.blocks(0)["resident"] and o.t.blocks(2)["resident"] and not o.t.blocks(1)["resident"]
    o.check()
    # after an eager pass over request 2 the same rotation fits
    assert o.eager(10) == 2
    o.rotate([0, 2], [1])
    o.check()


def test_hand_worked_allocation():
    """Lowest free id first, for blocks and for slots (readings of the table's policy)."""
    sh = W.KVShape(1, 1, 8, 4, n_hbm_blocks=6, n_host_slots=6)
    o = OracleSide(sh, O.BLOCK_FIRST)
    assert o.append(0, 5) == [0, 1]
    assert o.append(1, 4) == [2]
    assert o.append(0, 4) == [3]            # request 0 now 9 tokens: blocks 0, 1, 3
    assert o.eager(1) == 1                  # request 0's first full block -> slot 0
    assert o.t.blocks(0)["slots"] == [0, -1, -1]
    assert o.eager(10) == 2                 # request 0 block 1 -> slot 1, request 1 block 0 -> slot 2
    assert o.t.blocks(0)["slots"] == [0, 1, -1] and o.t.blocks(1)["slots"] == [2]
    o.finish(1)                             # frees HBM block 2 and slot 2
    assert o.append(2, 1) == [2]            # lowest free HBM block again
    o.rotate([0], [])                       # tail of request 0 -> lowest free slot, 2
    assert o.t.blocks(0)["slots"] == [0, 1, 2] and o.t.blocks(0)["ids"] == [-1, -1, -1]
    o.rotate([], [0])                       # back: lowest free HBM blocks 0, 1, 3
    assert o.t.blocks(0)["ids"] == [0, 1, 3]
    o.check()


def test_errors_change_nothing():
    o = OracleSide(SMALL, O.BLOCK_FIRST, max_req=4)
    o.append(0, 6)
    o.append(1, 6)
    snap = (o.cache.copy(), o.pool.copy(), o.t.counts(), o.t.blocks(0), o.t.blocks(1))
    o.rotate([2], [], expect=O.EINVAL)          # no such request
    o.rotate([0, 0], [], expect=O.EINVAL)       # named twice
    o.rotate([], [0], expect=O.EINVAL)          # resident request cannot be resumed
    o.rotate([7], [], expect=O.EINVAL)          # id out of range
    assert o.t.append(0, -1)[0] == O.EINVAL
    assert o.t.append(0, 1000)[0] == O.ENOSPC   # more blocks than the cache has
    assert o.t.finish(3) == O.EINVAL
    assert (o.t.counts(), o.t.blocks(0), o.t.blocks(1)) == snap[2:]
    assert np.array_equal(snap[0], o.cache) and np.array_equal(snap[1], o.pool)
    o.rotate([0], [])
    assert o.t.append(0, 1)[0] == O.EINVAL      # a rotary request cannot generate
    o.rotate([1], [0])
    o.check()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_schedules_preserve_every_token(layout, seed):
    """Random append / eager / rotate / finish sequences: after every step each
    request's tokens are readable through the table, synced blocks have valid
    DRAM copies, nothing is owned twice, free counts add up."""
    sh = W.KVShape(2, 2, 8, 4, n_hbm_blocks=24, n_host_slots=40)
    o = OracleSide(sh, layout, max_req=6, seed=seed)
    rng = np.random.default_rng(100 + seed)
    for step in range(160):
        op = rng.integers(0, 10)
        reqs = list(o.model.tokens)
        resident = [r for r in reqs if o.t.blocks(r)["resident"]]
        rotary = [r for r in reqs if not o.t.blocks(r)["resident"]]
        if op <= 3:
            cand = resident + [r for r in range(6) if r not in reqs]
            if cand:
                r = int(rng.choice(cand))
                n = int(rng.integers(0, 11))
                rc, _ = o.t.append(r, 0)
                need = -(-((o.t.blocks(r)["len"] if o.t.blocks(r) else 0) + n) // sh.block_size) - \
                    (len(o.t.blocks(r)["ids"]) if o.t.blocks(r) else 0)
                o.append(r, n, expect=O.OK if need <= o.t.counts()["free_hbm"] else O.ENOSPC)
                if o.t.blocks(r) is not None and r not in o.model.tokens:
                    o.model.tokens[r] = np.zeros((0,) + o.model.token_dims(), np.uint16)
        elif op <= 5:
            o.eager(int(rng.integers(0, 5)))
        elif op <= 8:
            pre = [r for r in resident if rng.random() < 0.4]
            res = [r for r in rotary if rng.random() < 0.5]
            if rng.random() < 0.5:
                rc = o.t.rotate(o.u8(o.cache), o.u8(o.pool), pre, res)
            else:
                rc, _ = o.t.rotate_eager(o.u8(o.cache), o.u8(o.pool), pre, res, int(rng.integers(0, 6)))
            assert rc in (O.OK, O.ENOSPC)
        elif reqs:
            o.finish(int(rng.choice(reqs)))
        o.check()
    c = o.t.counts()
    assert c["copied_eager"] > 0 and c["copied_preempt"] > 0 and c["dropped_synced"] > 0 and c["swapped_in"] > 0


def test_rotation_with_eager_step_hand_worked():
    """okvt_rotate_eager against a result worked out by hand from the rules alone
    (blocks and slots are always the lowest-numbered free ones; a preempted
    request copies out what has no DRAM copy; the blocks it copies out are not
    reusable within the call; the eager step comes after the rotation and visits
    resident requests by ascending id, blocks by index).  4-token blocks, 16 HBM
    blocks, 24 slots.

      append(0, 9)      request 0 takes blocks 0 1 2           FULL FULL DIRTY
      append(1, 8)      request 1 takes blocks 3 4             FULL FULL
      rotate([1], [])   1 has no DRAM copies: 3 4 -> slots 0 1; blocks 3 4 free again
      append(2, 14)     request 2 takes blocks 3 4 5 6         FULL FULL FULL DIRTY
      rotate_eager([0], [1], budget 2)
        request 0 out:  0 1 2 -> slots 2 3 4 (three copies at preemption, nothing to drop)
        request 1 in:   slots 0 1 -> blocks 7 8 (0 1 2 are being copied out, 3..6 are in use)
        eager step:     request 1 is all SYNCED; request 2's first two FULL blocks,
                        3 and 4, -> slots 5 6 and become SYNCED; the budget is spent
    """
    sh = W.KVShape(2, 2, 8, 4, n_hbm_blocks=16, n_host_slots=24)
    o = OracleSide(sh, O.BLOCK_FIRST, seed=9)
    assert o.append(0, 9) == [0, 1, 2]
    assert o.append(1, 8) == [3, 4]
    o.rotate([1], [])
    assert o.append(2, 14) == [3, 4, 5, 6]
    cv = V.hbm_view(sh, o.cache)
    before = {b: cv[:, :, b].copy() for b in range(7)}
    pv = V.pool_view(sh, o.pool, O.BLOCK_FIRST)
    staged = {sl: pv[:, :, sl].copy() for sl in (0, 1)}
    rc, n = o.t.rotate_eager(o.u8(o.cache), o.u8(o.pool), [0], [1], 2)
    assert (rc, n) == (O.OK, 2)
    assert o.t.blocks(0) == dict(ids=[-1, -1, -1], slots=[2, 3, 4], states=[HOST] * 3, len=9, resident=False)
    assert o.t.blocks(1) == dict(ids=[7, 8], slots=[0, 1], states=[SYNCED] * 2, len=8, resident=True)
    assert o.t.blocks(2) == dict(ids=[3, 4, 5, 6], slots=[5, 6, -1, -1], states=[SYNCED, SYNCED, FULL, DIRTY],
                                 len=14, resident=True)
    assert o.t.counts() == dict(free_hbm=10, free_slots=17, copied_eager=2, copied_preempt=5, dropped_synced=0,
                                swapped_in=2)
    # the bytes went where the table says
    for blk_id, slot in ((0, 2), (1, 3), (2, 4), (3, 5), (4, 6)):
        assert np.array_equal(pv[:, :, slot], before[blk_id]), f"slot {slot} does not hold block {blk_id}"
    for slot, blk_id in ((0, 7), (1, 8)):
        assert np.array_equal(cv[:, :, blk_id], staged[slot]), f"block {blk_id} does not hold slot {slot}"
    for b in range(7):
        assert np.array_equal(cv[:, :, b], before[b])      # copies, not moves
    o.check()


def test_rotation_with_the_eager_step_riding_along():
    """Request 0 leaves, request 1 comes back, and request 2, which stays, gets its
    full blocks copied out in the same call: counted as eager copies, SYNCED
    afterwards, and the whole outcome is that of a rotation followed by an eager step."""
    sh = W.KVShape(2, 2, 8, 4, n_hbm_blocks=16, n_host_slots=24)
    a, b = OracleSide(sh, O.BLOCK_FIRST, seed=5), OracleSide(sh, O.BLOCK_FIRST, seed=5)
    for o in (a, b):
        o.append(0, 9)                      # 3 blocks, the last one partly filled
        o.append(1, 8)
        o.rotate([1], [])                   # request 1 waits in DRAM
        o.append(2, 14)                     # 4 blocks, 3 of them full, never synced
    rc, n = a.t.rotate_eager(a.u8(a.cache), a.u8(a.pool), [0], [1], 2)
    assert (rc, n) == (O.OK, 2)
    assert a.t.blocks(2)["states"] == [SYNCED, SYNCED, FULL, DIRTY]
    assert a.t.blocks(0)["states"] == [HOST] * 3 and a.t.blocks(1)["states"] == [SYNCED] * 2
    b.rotate([0], [1])
    assert b.eager(2) == 2
    assert a.t.counts() == b.t.counts()
    for r in range(3):
        assert a.t.blocks(r) == b.t.blocks(r)
    assert np.array_equal(a.cache, b.cache) and np.array_equal(a.pool, b.pool)
    a.check()
    # errors change nothing, and a negative budget is one
    snap = (a.cache.copy(), a.pool.copy(), a.t.counts())
    assert a.t.rotate_eager(a.u8(a.cache), a.u8(a.pool), [1], [0], -1)[0] == O.EINVAL
    assert a.t.rotate_eager(a.u8(a.cache), a.u8(a.pool), [0], [], 3)[0] == O.EINVAL   # 0 is not resident
    assert np.array_equal(snap[0], a.cache) and np.array_equal(snap[1], a.pool) and snap[2] == a.t.counts()
