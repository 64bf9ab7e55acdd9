"""The arithmetic by which an in-heavy rotation spreads its out tiles over its in
tiles, restated with the kernel's integer widths and checked for what it must
guarantee: every out tile is met exactly once, by the in tile at which the
fixed-point product steps, and no 64-bit product overflows.  (The kernel itself
is compared with the oracle byte for byte in the GPU tests; this covers the
sizes those cannot reach.)"""
import random

M64 = (1 << 64) - 1


def mix_q(out_tiles, in_tiles):
    """Host side: ceil(out_tiles * 2^32 / in_tiles), in 64 bits."""
    v = ((out_tiles << 32) + in_tiles - 1)
    assert v <= M64
    return v // in_tiles


def out_tile_of(t, q, out_tiles):
    """Device side, for in tile t: the out tile that rides along, or None."""
    a = (t * q) & M64
    assert a == t * q, "64-bit product overflowed"
    b = (a + q) & M64
    assert b == a + q
    s0 = a >> 32
    s1 = min(b >> 32, out_tiles)
    assert s0 < (1 << 32)
    return s0 if s1 > s0 else None


def test_every_out_tile_exactly_once_exhaustive_small():
    for in_tiles in list(range(2, 70)) + [127, 128, 129, 1000]:
        for out_tiles in range(1, in_tiles):
            q = mix_q(out_tiles, in_tiles)
            assert q <= 1 << 32
            seen = [out_tile_of(t, q, out_tiles) for t in range(in_tiles)]
            met = [s for s in seen if s is not None]
            assert met == list(range(out_tiles)), (in_tiles, out_tiles)


def test_large_counts_by_sampling_and_closed_form():
    rng = random.Random(20309)
    limit = 0x7FFFFFFF - 1          # the engine refuses tile counts from 0x7FFFFFFF on
    cases = [(limit - 1, limit), (1, limit), (limit // 2, limit), (3, 7), (limit - 5, limit - 3)]
    cases += [(rng.randrange(1, l), l) for l in (rng.randrange(2, limit) for _ in range(200))]
    for out_tiles, in_tiles in cases:
        q = mix_q(out_tiles, in_tiles)
        assert 0 < q <= 1 << 32
        # the product steps by 0 or 1 per in tile and reaches out_tiles by the last one
        assert (in_tiles * q) >> 32 >= out_tiles
        assert ((in_tiles - 1) * q) >> 32 <= out_tiles
        # sampled in tiles: what rides along is the count of steps so far, and steps are 0 or 1
        for t in [0, 1, in_tiles - 1, in_tiles - 2] + [rng.randrange(in_tiles) for _ in range(50)]:
            if t < 0:
                continue
            s = out_tile_of(t, q, out_tiles)
            lo, hi = (t * q) >> 32, ((t + 1) * q) >> 32
            assert hi - lo in (0, 1)
            if s is not None:
                assert s == lo < out_tiles
            else:
                assert hi == lo or lo >= out_tiles
        # the last out tile is met by some in tile (binary search for the step to out_tiles)
        lo_t, hi_t = 0, in_tiles
        while lo_t < hi_t:
            mid = (lo_t + hi_t) // 2
            if ((mid + 1) * q) >> 32 >= out_tiles:
                hi_t = mid
            else:
                lo_t = mid + 1
        assert lo_t < in_tiles and out_tile_of(lo_t, q, out_tiles) == out_tiles - 1
