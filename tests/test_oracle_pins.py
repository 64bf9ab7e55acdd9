"""Pins for the CPU oracle: each check reaches the expected bytes by a route
that does not pass through the oracle's own offset or copy code."""
import itertools
import os

import numpy as np
import pytest

from oracle import kv_oracle as O
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V

LAYOUTS = [O.BLOCK_FIRST, O.LAYER_FIRST]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                out[k.strip()] = int(v)
    return out


def u8(a):
    return a.view(np.uint8)


def run_oracle(shape, layout, cache, pool, rot):
    s = O.shape_of(shape, layout)
    c, p = cache.copy(), pool.copy()
    rc = O.rotate(s, u8(c), u8(p), rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
    return rc, c, p


# ---- 5. sizes printed in the paper (Section 4.3.1 and Section 5.4, Table 2) ----

def test_sizes_match_paper_worked_example():
    g = read_golden("paper_worked_sizes.txt")
    s = O.make_shape(g["n_layers"], g["n_kv_heads"], g["head_dim"], g["block_size"],
                     n_hbm_blocks=4, n_host_slots=4, elem_bytes=g["elem_bytes"])
    # the paper's segment holds K and V of one layer-block; here they are two planes
    assert 2 * O.seg_bytes(s) == g["segment_k_plus_v"]
    assert O.block_bytes(s) == g["block_all_layers"]
    per_token = O.block_bytes(s) // g["block_size"]
    assert per_token == g["n_layers"] * g["per_token_per_layer_kv"]
    assert per_token * g["tokens_per_direction"] == g["bytes_per_direction"]
    # 32768 tokens are a whole number of 16-token blocks: 2048 of them
    assert g["tokens_per_direction"] % g["block_size"] == 0
    blocks = g["tokens_per_direction"] // g["block_size"]
    assert blocks == 2048 and blocks * O.block_bytes(s) == g["bytes_per_direction"]


def test_table2_e2e_definition():
    """Serial rows: E2E is the sum of the two one-way times at 8 'GB' each; the
    ideal row is 8/192.  Pins how end-to-end time is defined for the benchmark."""
    rows = {}
    with open(os.path.join(GOLDEN, "paper_table2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, d2h, h2d, e2e, mode = [x.strip() for x in line.split(",")]
            rows[name] = (float(d2h), float(h2d), float(e2e), mode)
    for name in ("naive", "ms", "ms_mk"):
        d2h, h2d, e2e, mode = rows[name]
        assert mode == "u"
        assert abs((8 / d2h + 8 / h2d) * 1e3 - e2e) / e2e < 2e-3
    d2h, h2d, e2e, _ = rows["ideal"]
    assert abs(8 / d2h * 1e3 - e2e) < 0.02
    d2h, h2d, e2e, _ = rows["duplexkv"]
    assert e2e >= max(8 / d2h, 8 / h2d) * 1e3  # wall time covers both streams


def test_sizes_of_configs():
    for name, seg, blk in [("tiny", 4096, 16384), ("llama3_8b", 32768, 2 << 20),
                           ("long70b", 65536, 10 << 20)]:
        s = O.shape_of(W.SHAPES[name])
        assert O.seg_bytes(s) == seg and O.block_bytes(s) == blk
        assert O.cache_bytes(s) == blk * W.SHAPES[name].n_hbm_blocks
        assert O.pool_bytes(s) == blk * W.SHAPES[name].n_host_slots


# ---- 1. brute force, element by element ----

def elem_off_hbm(sh, l, kv, b, t, h, d):
    return (((((l * 2 + kv) * sh.n_hbm_blocks + b) * sh.block_size + t) * sh.n_kv_heads + h)
            * sh.head_dim + d)


def elem_off_pool(sh, layout, l, kv, s, t, h, d):
    if layout == O.LAYER_FIRST:
        return (((((l * 2 + kv) * sh.n_host_slots + s) * sh.block_size + t) * sh.n_kv_heads + h)
                * sh.head_dim + d)
    return (((((s * sh.n_layers + l) * 2 + kv) * sh.block_size + t) * sh.n_kv_heads + h)
            * sh.head_dim + d)


def brute_force(sh, layout, cache, pool, rot):
    c, p = cache.copy(), pool.copy()
    idx = lambda: itertools.product(range(sh.n_layers), range(2), range(sh.block_size),
                                    range(sh.n_kv_heads), range(sh.head_dim))
    for b, s in zip(rot.out_ids, rot.out_slots):
        for l, kv, t, h, d in idx():
            p[elem_off_pool(sh, layout, l, kv, int(s), t, h, d)] = \
                cache[elem_off_hbm(sh, l, kv, int(b), t, h, d)]
    for b, s in zip(rot.in_ids, rot.in_slots):
        for l, kv, t, h, d in idx():
            c[elem_off_hbm(sh, l, kv, int(b), t, h, d)] = \
                pool[elem_off_pool(sh, layout, l, kv, int(s), t, h, d)]
    return c, p


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_brute_force_six_loops(name, layout):
    sh = W.SHAPES[name]
    rot = W.config_rotation(name)
    if name == "tiny":  # keep the Python loops short: 3 out, 3 in
        rot = W.Rotation(rot.out_ids[:3], rot.out_slots[:3], rot.in_ids[:3], rot.in_slots[:3])
    cache, pool = V.make_images(sh, layout, rot, W.value_seed(name))
    rc, c, p = run_oracle(sh, layout, cache, pool, rot)
    assert rc == O.OK
    cb, pb = brute_force(sh, layout, cache, pool, rot)
    assert np.array_equal(c, cb) and np.array_equal(p, pb)
    assert not np.array_equal(c, cache) and not np.array_equal(p, pool)


# ---- 2. tagged fill: closed form of every byte after the rotation ----

def tag(l, kv, blk, t, h, d):
    """16-bit tag of element (l,kv,t,h,d) of logical block `blk` (NumPy broadcastable)."""
    x = (np.uint64(0x9E3779B97F4A7C15) * (np.asarray(blk, dtype=np.uint64) + np.uint64(1))
         + np.uint64(0xBF58476D1CE4E5B9) * np.asarray(l, dtype=np.uint64)
         + np.uint64(0x94D049BB133111EB) * np.asarray(kv, dtype=np.uint64)
         + np.uint64(0x2545F4914F6CDD1D) * np.asarray(t, dtype=np.uint64)
         + np.uint64(0xD6E8FEB86659FD93) * np.asarray(h, dtype=np.uint64)
         + np.uint64(0xCA5A826395121157) * np.asarray(d, dtype=np.uint64))
    x ^= x >> np.uint64(29)
    return ((x >> np.uint64(13)) & np.uint64(0xFFFF)).astype(np.uint16)


def tagged_images(sh, layout):
    """cache block b holds tags of logical block b; pool slot s holds tags of logical
    block NB + s."""
    L, P, H, D = sh.n_layers, sh.block_size, sh.n_kv_heads, sh.head_dim
    g = np.ix_(np.arange(L), np.arange(2), np.arange(1), np.arange(P), np.arange(H), np.arange(D))
    l, kv, _, t, h, d = g
    cache = np.empty(V.n_cache_elems(sh), dtype=np.uint16)
    pool = np.empty(V.n_pool_elems(sh), dtype=np.uint16)
    cv, pv = V.hbm_view(sh, cache), V.pool_view(sh, pool, layout)
    with np.errstate(over="ignore"):
        for b in range(sh.n_hbm_blocks):
            cv[:, :, b:b + 1] = tag(l, kv, b, t, h, d)
        for s in range(sh.n_host_slots):
            pv[:, :, s:s + 1] = tag(l, kv, sh.n_hbm_blocks + s, t, h, d)
    return cache, pool


def tagged_ok(sh, layout, c, p, rot):
    """True iff (c, p) is what the rotation must leave behind, from tags alone."""
    L, P, H, D = sh.n_layers, sh.block_size, sh.n_kv_heads, sh.head_dim
    l, kv, _, t, h, d = np.ix_(np.arange(L), np.arange(2), np.arange(1), np.arange(P),
                               np.arange(H), np.arange(D))
    cv, pv = V.hbm_view(sh, c), V.pool_view(sh, p, layout)
    logical_in_block = {int(b): sh.n_hbm_blocks + int(s) for b, s in zip(rot.in_ids, rot.in_slots)}
    logical_in_slot = {int(s): int(b) for b, s in zip(rot.out_ids, rot.out_slots)}
    with np.errstate(over="ignore"):
        for b in range(sh.n_hbm_blocks):
            if not np.array_equal(cv[:, :, b:b + 1], tag(l, kv, logical_in_block.get(b, b), t, h, d)):
                return False
        for s in range(sh.n_host_slots):
            want = logical_in_slot.get(s, sh.n_hbm_blocks + s)
            if not np.array_equal(pv[:, :, s:s + 1], tag(l, kv, want, t, h, d)):
                return False
    return True


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_tagged_fill_closed_form(name, layout):
    sh = W.SHAPES[name]
    rot = W.config_rotation(name)
    cache, pool = tagged_images(sh, layout)
    rc, c, p = run_oracle(sh, layout, cache, pool, rot)
    assert rc == O.OK
    assert tagged_ok(sh, layout, c, p, rot)


@pytest.mark.parametrize("layout", LAYOUTS)
def test_tagged_check_catches_planted_mistakes(layout):
    """The closed-form check must reject the plausible wrong answers."""
    sh = W.SHAPES["tiny"]
    rot = W.config_rotation("tiny")
    cache, pool = tagged_images(sh, layout)
    rc, c, p = run_oracle(sh, layout, cache, pool, rot)
    assert tagged_ok(sh, layout, c, p, rot)
    # K and V planes exchanged in the pool copy of one block
    p1 = p.copy(); pv = V.pool_view(sh, p1, layout); s0 = int(rot.out_slots[0])
    pv[:, :, s0] = pv[:, ::-1, s0].copy()
    assert not tagged_ok(sh, layout, c, p1, rot)
    # last layer of one swapped-in block never written
    c1 = c.copy(); cv = V.hbm_view(sh, c1); b0 = int(rot.in_ids[-1])
    cv[-1, :, b0] = V.hbm_view(sh, cache)[-1, :, b0]
    assert not tagged_ok(sh, layout, c1, p, rot)
    # ids paired with the wrong slots (rotated by one)
    wrong = W.Rotation(rot.out_ids, np.roll(rot.out_slots, 1), rot.in_ids, rot.in_slots)
    rc, c2, p2 = run_oracle(sh, layout, cache, pool, wrong)
    assert not tagged_ok(sh, layout, c2, p2, rot)
    # one stray element in an un-named block
    c3 = c.copy(); named = set(rot.in_ids.tolist()) | set(rot.out_ids.tolist())
    other = next(b for b in range(sh.n_hbm_blocks) if b not in named)
    V.hbm_view(sh, c3)[0, 1, other, 3, 1, 7] ^= 1
    assert not tagged_ok(sh, layout, c3, p, rot)
    # the other host layout's answer is not accepted for this layout
    rc, c4, p4 = run_oracle(sh, 1 - layout, cache, pool, rot)
    assert not tagged_ok(sh, layout, c4, p4, rot)


# ---- 4. the rotation as array indexing (library routine) ----

@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged", "small8b"])
def test_equals_numpy_indexing(name, layout):
    sh = W.SHAPES[name]
    rot = W.config_rotation(name)
    cache, pool = V.make_images(sh, layout, rot, W.value_seed(name))
    rc, c, p = run_oracle(sh, layout, cache, pool, rot)
    assert rc == O.OK
    ce, pe = V.expected_by_indexing(sh, layout, cache, pool, rot)
    assert np.array_equal(c, ce) and np.array_equal(p, pe)


def test_equals_numpy_indexing_llama_planes():
    """Llama-3-8B plane shape (32 layers, 32 KiB segments) on a cut-down block count."""
    import dataclasses
    sh = dataclasses.replace(W.SHAPES["llama3_8b"], n_hbm_blocks=48, n_host_slots=40)
    rot = W.simple_rotation(sh, 16, 16, seed=5)
    for layout in LAYOUTS:
        cache, pool = V.make_images(sh, layout, rot, 77)
        rc, c, p = run_oracle(sh, layout, cache, pool, rot)
        assert rc == O.OK
        ce, pe = V.expected_by_indexing(sh, layout, cache, pool, rot)
        assert np.array_equal(c, ce) and np.array_equal(p, pe)


# ---- 3. invariants ----

@pytest.mark.parametrize("layout", LAYOUTS)
def test_round_trip_is_identity_and_permutation(layout):
    sh = W.SHAPES["tiny"]
    rot = W.config_rotation("tiny")
    cache, pool = V.make_images(sh, layout, rot, 1)
    s = O.shape_of(sh, layout)
    c, p = cache.copy(), pool.copy()
    # out, then in to the same ids: cache unchanged
    assert O.swap_out(s, u8(c), u8(p), rot.out_ids, rot.out_slots) == O.OK
    assert np.array_equal(c, cache)            # source bytes are not cleared
    c[...] = 0
    assert O.swap_in(s, u8(c), u8(p), rot.out_slots, rot.out_ids) == O.OK
    cv, cv0 = V.hbm_view(sh, c), V.hbm_view(sh, cache)
    assert np.array_equal(cv[:, :, rot.out_ids], cv0[:, :, rot.out_ids])
    mask = np.ones(sh.n_hbm_blocks, bool); mask[rot.out_ids] = False
    assert not cv[:, :, mask].any()            # nothing else was written
    # out to slots S, in from S to other ids B: block permutation
    c = cache.copy(); p = pool.copy()
    O.swap_out(s, u8(c), u8(p), rot.out_ids, rot.out_slots)
    O.swap_in(s, u8(c), u8(p), rot.out_slots, rot.in_ids)
    cv = V.hbm_view(sh, c)
    assert np.array_equal(cv[:, :, rot.in_ids], cv0[:, :, rot.out_ids])


@pytest.mark.parametrize("layout", LAYOUTS)
def test_unnamed_untouched_idempotent_and_sequential_equivalence(layout):
    sh = W.SHAPES["tiny"]
    rot = W.config_rotation("tiny")
    cache, pool = V.make_images(sh, layout, rot, 2)
    s = O.shape_of(sh, layout)
    rc, c, p = run_oracle(sh, layout, cache, pool, rot)
    cv, cv0 = V.hbm_view(sh, c), V.hbm_view(sh, cache)
    pv, pv0 = V.pool_view(sh, p, layout), V.pool_view(sh, pool, layout)
    bm = np.ones(sh.n_hbm_blocks, bool); bm[rot.in_ids] = False
    sm = np.ones(sh.n_host_slots, bool); sm[rot.out_slots] = False
    assert np.array_equal(cv[:, :, bm], cv0[:, :, bm])
    assert np.array_equal(pv[:, :, sm], pv0[:, :, sm])
    # swap_out twice leaves the same pool
    c1, p1 = cache.copy(), pool.copy()
    O.swap_out(s, u8(c1), u8(p1), rot.out_ids, rot.out_slots)
    p_once = p1.copy()
    O.swap_out(s, u8(c1), u8(p1), rot.out_ids, rot.out_slots)
    assert np.array_equal(p1, p_once)
    # rotate == swap_out then swap_in == swap_in then swap_out
    for order in (0, 1):
        c2, p2 = cache.copy(), pool.copy()
        steps = [lambda: O.swap_out(s, u8(c2), u8(p2), rot.out_ids, rot.out_slots),
                 lambda: O.swap_in(s, u8(c2), u8(p2), rot.in_slots, rot.in_ids)]
        for f in (steps if order == 0 else steps[::-1]):
            assert f() == O.OK
        assert np.array_equal(c2, c) and np.array_equal(p2, p)
    # threaded split gives the same bytes
    for threads in (1, 3, 8):
        c3, p3 = cache.copy(), pool.copy()
        assert O.rotate(s, u8(c3), u8(p3), rot.out_ids, rot.out_slots, rot.in_ids,
                        rot.in_slots, threads=threads) == O.OK
        assert np.array_equal(c3, c) and np.array_equal(p3, p)
    # a rotation followed by its inverse restores cache blocks and pool slots that it named
    c4, p4 = c.copy(), p.copy()
    inv = rot.inverse()
    assert O.rotate(s, u8(c4), u8(p4), inv.out_ids, inv.out_slots, inv.in_ids, inv.in_slots) == O.OK
    assert np.array_equal(V.hbm_view(sh, c4)[:, :, rot.out_ids], cv0[:, :, rot.out_ids])
    assert np.array_equal(V.pool_view(sh, p4, layout)[:, :, rot.in_slots], pv0[:, :, rot.in_slots])


def test_empty_and_full_lists():
    sh = W.SHAPES["tiny"]
    s = O.shape_of(sh)
    rot = W.config_rotation("tiny")
    cache, pool = V.make_images(sh, O.BLOCK_FIRST, rot, 3)
    c, p = cache.copy(), pool.copy()
    assert O.rotate(s, u8(c), u8(p), None, None, None, None) == O.OK
    assert O.rotate(s, u8(c), u8(p), [], [], [], []) == O.OK
    assert np.array_equal(c, cache) and np.array_equal(p, pool)
    # every slot filled from distinct blocks: the largest swap-out this pool admits
    ids = np.arange(sh.n_host_slots, dtype=np.int32)[::-1] + 5
    slots = np.arange(sh.n_host_slots, dtype=np.int32)
    assert O.swap_out(s, u8(c), u8(p), ids, slots) == O.OK
    pv = V.pool_view(sh, p, O.BLOCK_FIRST)
    assert np.array_equal(pv[:, :, slots], V.hbm_view(sh, cache)[:, :, ids])


# ---- admission rules ----

def expected_code(sh, oi, os_, ii, is_):
    """The admission rules restated with Python sets, in the fixed order."""
    lists = [(oi, sh.n_hbm_blocks), (os_, sh.n_host_slots), (ii, sh.n_hbm_blocks),
             (is_, sh.n_host_slots)]
    if any(x < 0 or x >= lim for lst, lim in lists for x in lst):
        return O.ERANGE
    if any(len(set(lst)) != len(lst) for lst, _ in lists):
        return O.EDUP
    if set(oi) & set(ii) or set(os_) & set(is_):
        return O.EOVERLAP
    return O.OK


def test_validate_matches_set_logic_on_random_lists():
    sh = W.KVShape(1, 1, 8, 2, n_hbm_blocks=9, n_host_slots=7)
    s = O.shape_of(sh)
    rng = np.random.default_rng(12)
    seen = set()
    for _ in range(4000):
        no, ni = rng.integers(0, 4, size=2)
        oi = rng.integers(-1, sh.n_hbm_blocks + 1, size=no).tolist()
        os_ = rng.integers(-1, sh.n_host_slots + 1, size=no).tolist()
        ii = rng.integers(-1, sh.n_hbm_blocks + 1, size=ni).tolist()
        is_ = rng.integers(-1, sh.n_host_slots + 1, size=ni).tolist()
        want = expected_code(sh, oi, os_, ii, is_)
        assert O.validate(s, oi, os_, ii, is_) == want
        seen.add(want)
    assert seen == {O.OK, O.ERANGE, O.EDUP, O.EOVERLAP}


REJECTS = [
    # (out_ids, out_slots, in_ids, in_slots, code)
    ([64], [0], [], [], O.ERANGE),            # block id == NB
    ([-1], [0], [], [], O.ERANGE),            # padding value of a 2-D block table
    ([0], [32], [], [], O.ERANGE),            # slot == NS
    ([], [], [0], [-5], O.ERANGE),
    ([3, 3], [0, 1], [], [], O.EDUP),         # duplicate source block
    ([3, 4], [1, 1], [], [], O.EDUP),         # duplicate destination slot
    ([], [], [7, 7], [0, 1], O.EDUP),         # duplicate destination block
    ([], [], [7, 8], [2, 2], O.EDUP),         # duplicate source slot
    ([5], [0], [5], [1], O.EOVERLAP),         # swap-in lands on a swap-out source
    ([5], [4], [6], [4], O.EOVERLAP),         # a slot read and written in one call
    ([5, 64], [0, 0], [5], [1], O.ERANGE),    # range outranks duplicate and overlap
    ([5, 6], [0, 0], [5], [1], O.EDUP),       # duplicate outranks overlap
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("case", REJECTS)
def test_rejections_touch_nothing(case, layout):
    sh = W.SHAPES["tiny"]
    s = O.shape_of(sh, layout)
    rot = W.config_rotation("tiny")
    cache, pool = V.make_images(sh, layout, rot, 4)
    c, p = cache.copy(), pool.copy()
    oi, os_, ii, is_, code = case
    assert O.rotate(s, u8(c), u8(p), oi, os_, ii, is_) == code
    assert np.array_equal(c, cache) and np.array_equal(p, pool)


def test_einval():
    sh = W.SHAPES["tiny"]
    s = O.shape_of(sh)
    assert O.validate(s, None, None, None, None, n_out=-1) == O.EINVAL
    assert O.validate(s, None, None, None, None, n_out=2) == O.EINVAL   # NULL with n > 0
    assert O.validate(s, None, None, None, None, n_in=1) == O.EINVAL
    bad = O.make_shape(0, 2, 64, 16, 64, 32)
    assert O.validate(bad, [1], [1], None, None) == O.EINVAL
    bad = O.make_shape(2, 2, 64, 16, 64, 32, host_layout=2)
    assert O.validate(bad, [1], [1], None, None) == O.EINVAL
    c = np.zeros(O.cache_bytes(s), np.uint8)
    assert O.rotate(s, c, None, [1], [1], None, None) == O.EINVAL       # NULL pool


def test_offsets_are_a_bijection_onto_the_images():
    """Every segment offset is distinct, aligned to the segment size and inside the image."""
    sh = W.SHAPES["ragged"]
    for layout in LAYOUTS:
        s = O.shape_of(sh, layout)
        seg = O.seg_bytes(s)
        h = {O.hbm_offset(s, l, kv, b) for l in range(sh.n_layers) for kv in range(2)
             for b in range(sh.n_hbm_blocks)}
        p = {O.pool_offset(s, l, kv, sl) for l in range(sh.n_layers) for kv in range(2)
             for sl in range(sh.n_host_slots)}
        assert h == set(range(0, O.cache_bytes(s), seg))
        assert p == set(range(0, O.pool_bytes(s), seg))


# ---- decode reader checksum ----

@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_read_checksum_against_numpy_and_closed_form(name):
    sh = W.SHAPES[name]
    s = O.shape_of(sh)
    rot = W.config_rotation(name)
    cache, _ = V.make_images(sh, O.BLOCK_FIRST, rot, 9)
    ids = np.concatenate([rot.out_ids, rot.in_ids])
    rc, got = O.read_checksum(s, u8(cache), ids)
    assert rc == O.OK
    # library routine: gather the blocks by indexing, view as little-endian words, sum
    blocks = np.ascontiguousarray(V.hbm_view(sh, cache)[:, :, ids])
    want = int(blocks.view("<u4").sum(dtype=np.uint64))
    assert got == want
    # closed form: a constant fill makes the sum words x constant (and it wraps mod 2^64)
    const = np.full_like(cache, 0xFFFF)
    rc, got = O.read_checksum(s, u8(const), ids)
    words = len(ids) * O.block_bytes(s) // 4
    assert got == (words * 0xFFFFFFFF) % (1 << 64)
    # one flipped bit anywhere in a named block moves the sum by exactly that bit
    c2 = cache.copy()
    V.hbm_view(sh, c2)[sh.n_layers - 1, 1, int(ids[-1]), sh.block_size - 1, 0, 1] ^= 0x0100
    rc, got2 = O.read_checksum(s, u8(c2), ids)
    rc, got1 = O.read_checksum(s, u8(cache), ids)
    assert (got2 - got1) % (1 << 64) in (0x0100_0000 % (1 << 64), (-0x0100_0000) % (1 << 64))
    # an un-named block does not enter
    other = next(b for b in range(sh.n_hbm_blocks) if b not in set(ids.tolist()))
    c3 = cache.copy(); V.hbm_view(sh, c3)[:, :, other] ^= 0xFFFF
    assert O.read_checksum(s, u8(c3), ids)[1] == got1
    # a block named twice counts twice; order does not matter; empty list sums to 0
    rc, twice = O.read_checksum(s, u8(cache), np.concatenate([ids, ids[::-1]]))
    assert twice == (2 * got1) % (1 << 64)
    assert O.read_checksum(s, u8(cache), [])[1] == 0
    assert O.read_checksum(s, u8(cache), [sh.n_hbm_blocks])[0] == O.ERANGE


# ---- block-first cache layout (Section 4.3.2, "Block-first layout and batched KV transfers") ----

def elem_off_hbm_block_first(sh, l, kv, b, t, h, d):
    return (((((b * sh.n_layers + l) * 2 + kv) * sh.block_size + t) * sh.n_kv_heads + h)
            * sh.head_dim + d)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged"])
def test_block_first_cache_brute_force_and_indexing(name, layout):
    sh = W.SHAPES[name]
    rot = W.config_rotation(name)
    if name == "tiny":
        rot = W.Rotation(rot.out_ids[:3], rot.out_slots[:3], rot.in_ids[:3], rot.in_slots[:3])
    cache, pool = V.make_images(sh, layout, rot, W.value_seed(name), hbm_layout=1)
    s = O.shape_of(sh, layout, O.HBM_BLOCK_FIRST)
    c, p = cache.copy(), pool.copy()
    assert O.rotate(s, u8(c), u8(p), rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots) == O.OK
    # six loops over elements, with the block-first element offset written out
    cb, pb = cache.copy(), pool.copy()
    idx = lambda: itertools.product(range(sh.n_layers), range(2), range(sh.block_size),
                                    range(sh.n_kv_heads), range(sh.head_dim))
    for b, sl in zip(rot.out_ids, rot.out_slots):
        for l, kv, t, h, d in idx():
            pb[elem_off_pool(sh, layout, l, kv, int(sl), t, h, d)] = \
                cache[elem_off_hbm_block_first(sh, l, kv, int(b), t, h, d)]
    for b, sl in zip(rot.in_ids, rot.in_slots):
        for l, kv, t, h, d in idx():
            cb[elem_off_hbm_block_first(sh, l, kv, int(b), t, h, d)] = \
                pool[elem_off_pool(sh, layout, l, kv, int(sl), t, h, d)]
    assert np.array_equal(c, cb) and np.array_equal(p, pb)
    # the same through array indexing on the block-first view
    ce, pe = V.expected_by_indexing(sh, layout, cache, pool, rot, hbm_layout=1)
    assert np.array_equal(c, ce) and np.array_equal(p, pe)
    # and it is not what the layer-first reading of the same bytes gives
    s0 = O.shape_of(sh, layout, O.HBM_LAYER_FIRST)
    c0, p0 = cache.copy(), pool.copy()
    O.rotate(s0, u8(c0), u8(p0), rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots)
    assert not np.array_equal(p0, p)


def test_block_first_cache_strides_match_the_paper():
    """With the block-first layout the stride between blocks i and j is
    (j - i) x N_L x S_seg and a block is one contiguous region (4 MB for the
    worked example); with the layer-first layout it is (j - i) x S_seg."""
    g = read_golden("paper_worked_sizes.txt")
    for hbm_layout, stride in [(O.HBM_BLOCK_FIRST, g["n_layers"] * g["segment_k_plus_v"]),
                               (O.HBM_LAYER_FIRST, g["segment_k_plus_v"] // 2)]:
        s = O.make_shape(g["n_layers"], g["n_kv_heads"], g["head_dim"], g["block_size"], 16, 16,
                         elem_bytes=g["elem_bytes"], hbm_layout=hbm_layout)
        assert O.hbm_offset(s, 0, 0, 7) - O.hbm_offset(s, 0, 0, 3) == 4 * stride
    s = O.make_shape(g["n_layers"], g["n_kv_heads"], g["head_dim"], g["block_size"], 16, 16,
                     elem_bytes=g["elem_bytes"], hbm_layout=O.HBM_BLOCK_FIRST)
    offs = sorted(O.hbm_offset(s, l, kv, 5) for l in range(g["n_layers"]) for kv in range(2))
    assert offs[0] == 5 * g["block_all_layers"]
    assert offs == list(range(offs[0], offs[0] + g["block_all_layers"], O.seg_bytes(s)))
    # offsets still tile the image exactly
    sh = W.SHAPES["ragged"]
    s = O.shape_of(sh, O.BLOCK_FIRST, O.HBM_BLOCK_FIRST)
    h = {O.hbm_offset(s, l, kv, b) for l in range(sh.n_layers) for kv in range(2) for b in range(sh.n_hbm_blocks)}
    assert h == set(range(0, O.cache_bytes(s), O.seg_bytes(s)))


def test_block_first_cache_checksum_and_bad_layout():
    sh = W.SHAPES["ragged"]
    rot = W.config_rotation("ragged")
    cache, _ = V.make_images(sh, O.BLOCK_FIRST, rot, 9, hbm_layout=1)
    s = O.shape_of(sh, O.BLOCK_FIRST, O.HBM_BLOCK_FIRST)
    ids = np.concatenate([rot.out_ids, rot.in_ids])
    rc, got = O.read_checksum(s, u8(cache), ids)
    blocks = np.ascontiguousarray(V.hbm_view(sh, cache, 1)[:, :, ids])
    assert rc == O.OK and got == int(blocks.view("<u4").sum(dtype=np.uint64))
    bad = O.make_shape(2, 2, 64, 16, 64, 32, hbm_layout=2)
    assert O.validate(bad, [1], [1], None, None) == O.EINVAL
