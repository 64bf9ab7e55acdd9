"""Parity of the HIP path with the CPU oracle, through the C ABI, bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests.gpu_harness import GpuCase, make_case
from tests import kvviews as V

pytestmark = pytest.mark.gpu

LAYOUTS = [B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST]
PATHS = [B.KV_PATH_AUTO, B.KV_PATH_FUSED, B.KV_PATH_ZEROCOPY, B.KV_PATH_SDMA_STAGED, B.KV_PATH_NAIVE]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged", "small8b"])
def test_rotate_matches_oracle(name, layout, path):
    case, rot = make_case(name, layout, path)
    case.rotate(rot)
    case.check()
    st = case.eng.kv_last_stats()
    blk = B.kv_block_bytes(case.cfg)
    assert st["bytes_out"] == len(rot.out_ids) * blk and st["bytes_in"] == len(rot.in_ids) * blk
    # and back again: the inverse rotation restores the named blocks
    case.rotate(rot.inverse())
    case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_SDMA_STAGED, B.KV_PATH_NAIVE])
@pytest.mark.parametrize("layout", LAYOUTS)
def test_single_directions_and_round_trip(layout, path):
    case, rot = make_case("small8b", layout, path)
    case.swap_out(rot.out_ids, rot.out_slots)
    case.check()
    case.swap_in(rot.in_slots, rot.in_ids)
    case.check()
    # the swapped-out copies come back: first into their own blocks (identity) ...
    case.swap_in(rot.out_slots, rot.out_ids)
    case.check()
    # ... then into other blocks (a block permutation)
    n = min(len(rot.out_slots), len(rot.in_ids))
    case.swap_in(rot.out_slots[:n], rot.in_ids[:n][::-1].copy())
    case.check()
    case.close()


@pytest.mark.parametrize("path", PATHS)
def test_unbalanced_empty_and_one_block(path):
    sh = W.SHAPES["small8b"]
    for n_out, n_in in [(40, 3), (3, 40), (1, 1), (0, 5), (5, 0), (0, 0)]:
        rot = W.simple_rotation(sh, n_out, n_in, seed=n_out * 100 + n_in)
        case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, path, rot=rot)
        case.rotate(rot)
        case.check()
        case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY, B.KV_PATH_SDMA_STAGED])
@pytest.mark.parametrize("layout", LAYOUTS)
def test_maximum_lists(layout, path):
    """Every host slot in use: half filled from HBM, half emptied into it."""
    sh = W.SHAPES["tiny"]
    half = sh.n_host_slots // 2
    rot = W.simple_rotation(sh, half, half, seed=3, n_used=sh.n_hbm_blocks // 2)
    case, _ = make_case(sh, layout, path, rot=rot)
    case.rotate(rot)
    case.check()
    case.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_rejections_enqueue_nothing(layout):
    case, rot = make_case("tiny", layout, B.KV_PATH_AUTO)
    nb, ns = case.shape.n_hbm_blocks, case.shape.n_host_slots
    bad = [
        (W.Rotation(np.array([nb]), np.array([0]), np.array([], int), np.array([], int)), B.KV_ERANGE),
        (W.Rotation(np.array([0]), np.array([-1]), np.array([], int), np.array([], int)), B.KV_ERANGE),
        (W.Rotation(np.array([3, 3]), np.array([0, 1]), np.array([], int), np.array([], int)), B.KV_EDUP),
        (W.Rotation(np.array([], int), np.array([], int), np.array([7, 8]), np.array([2, 2])), B.KV_EDUP),
        (W.Rotation(np.array([5]), np.array([0]), np.array([5]), np.array([1])), B.KV_EOVERLAP),
        (W.Rotation(np.array([5]), np.array([4]), np.array([6]), np.array([4])), B.KV_EOVERLAP),
        (W.Rotation(np.array([5, 6]), np.array([0, 0]), np.array([5]), np.array([1])), B.KV_EDUP),
    ]
    for r, code in bad:
        case.rotate(r, expect=code)
    case.check()               # nothing moved
    case.rotate(rot)           # and the engine still works afterwards
    case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY, B.KV_PATH_SDMA_STAGED])
def test_many_calls_without_wait_wrap_the_descriptor_ring(path):
    sh = W.SHAPES["small8b"]
    rng = np.random.default_rng(8)
    perm = rng.permutation(sh.n_hbm_blocks).astype(np.int32)
    sperm = rng.permutation(sh.n_host_slots).astype(np.int32)
    rot0 = W.Rotation(perm[:0], sperm[:0], perm[:0], sperm[:0])
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, path, rot=rot0)
    # 20 disjoint small rotations back to back, more than the ring holds
    for c in range(20):
        o = perm[c * 6:c * 6 + 3]; i = perm[c * 6 + 3:c * 6 + 6]
        so = sperm[c * 6:c * 6 + 3]; si = sperm[c * 6 + 3:c * 6 + 6]
        case.rotate(W.Rotation(o, so, i, si))
    case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY, B.KV_PATH_SDMA_STAGED])
def test_caller_owned_pool_and_streams(path):
    case, rot = make_case("small8b", B.KV_HOST_LAYER_FIRST, path, own_pool=False, own_streams=False)
    case.rotate(rot)
    # work enqueued on the caller's in-stream afterwards sees the swapped-in blocks
    with torch.cuda.stream(case.streams[1]):
        snap = case.dev_cache.clone()
    case.check()
    assert torch.equal(snap.cpu(), case.dev_cache.cpu())
    case.close()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("chunk_layers,staging", [(0, 2 << 20), (1, 2 << 20), (2, 8 << 20), (0, 1 << 20)])
def test_staged_chunking_small_buffers(layout, chunk_layers, staging):
    """Staging far smaller than the rotation: many chunks, both buffers reused,
    plane ranges and block ranges split."""
    case, rot = make_case("small8b", layout, B.KV_PATH_SDMA_STAGED, chunk_layers=chunk_layers,
                          staging_bytes=staging)
    case.rotate(rot)
    case.check()
    assert case.eng.kv_last_stats()["n_launches"] > 4
    case.rotate(rot.inverse())
    case.check()
    case.close()


def test_staged_contiguous_slots_merge_into_few_copies():
    sh = W.SHAPES["small8b"]
    rot = W.simple_rotation(sh, 32, 32, seed=4, contiguous_slots=True)
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_SDMA_STAGED, rot=rot)
    case.rotate(rot)
    case.check()
    # 32 blocks x 256 KiB = 8 MiB per direction fits one chunk: 1 kernel + 1 copy each way
    assert case.eng.kv_last_stats()["n_launches"] == 4
    case.close()


@pytest.mark.parametrize("max_wgs", [1, 7, 64])
def test_workgroup_cap(max_wgs):
    case, rot = make_case("small8b", B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO, max_copy_wgs=max_wgs)
    case.rotate(rot)
    case.check()
    case.close()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,max_wgs,staging", [("small8b", 1, 0), ("small8b", 64, 2 << 20), ("ragged", 3, 0),
                                                  ("tiny", 2, 0)])
def test_staged_path_with_capped_workgroups(name, max_wgs, staging, layout):
    """With a cap on its workgroups the DMA-staged path packs and unpacks with
    persistent waves of the general move kernel instead of one wave per tile."""
    case, rot = make_case(name, layout, B.KV_PATH_SDMA_STAGED, max_copy_wgs=max_wgs, staging_bytes=staging)
    case.rotate(rot)
    case.check()
    case.rotate(rot.inverse())
    case.check()
    case.close()


def test_unaligned_segments_use_narrow_vectors():
    """Segment sizes that are not multiples of 16 bytes (2-byte and 1-byte lanes)."""
    for sh in [W.KVShape(2, 1, 3, 1, n_hbm_blocks=11, n_host_slots=9, elem_bytes=2),   # 6 B
               W.KVShape(2, 1, 7, 3, n_hbm_blocks=11, n_host_slots=9, elem_bytes=1),   # 21 B
               W.KVShape(2, 3, 5, 4, n_hbm_blocks=11, n_host_slots=9, elem_bytes=2)]:  # 120 B
        rot = W.simple_rotation(sh, 4, 3, seed=2)
        oshape = O.shape_of(sh, 0)
        rng = np.random.default_rng(3)
        cache = rng.integers(0, 256, O.cache_bytes(oshape), dtype=np.uint8)
        pool = rng.integers(0, 256, O.pool_bytes(oshape), dtype=np.uint8)
        if cache.size % 2:
            continue
        for path in (B.KV_PATH_AUTO, B.KV_PATH_SDMA_STAGED):
            case = GpuCase(sh, 0, path, cache.view(np.uint16), pool.view(np.uint16))
            case.rotate(rot)
            case.check()
            case.close()


def test_create_rejects_undersized_cache():
    sh = W.SHAPES["tiny"]
    cfg = B.make_config(sh)
    # a separate small allocation, not a slice of a larger one
    small = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    big_cfg = B.make_config(dataclasses.replace(sh, n_hbm_blocks=1 << 20))
    with pytest.raises(B.KVError) as ei:
        B.Engine(big_cfg, small.data_ptr())
    assert ei.value.code == B.KV_EINVAL
    with pytest.raises(B.KVError):
        B.Engine(cfg, small.data_ptr(), host_pool_ptr=small.data_ptr())   # pool must be host memory


@pytest.mark.parametrize("lanes", [64, 512, 1024])
def test_workgroup_width(lanes):
    """The move kernels take their tile width from the launch: any multiple of 64 lanes."""
    for name, path in [("ragged", B.KV_PATH_FUSED), ("small8b", B.KV_PATH_FUSED), ("small8b", B.KV_PATH_ZEROCOPY)]:
        case, rot = make_case(name, B.KV_HOST_BLOCK_FIRST, path, wg_lanes=lanes)
        case.rotate(rot)
        case.check()
        case.close()


BF = dict(hbm_layout=B.KV_HBM_BLOCK_FIRST)


@pytest.mark.parametrize("path", PATHS + [B.KV_PATH_DMA_BLOCKS])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["tiny", "ragged", "small8b"])
def test_block_first_cache(name, layout, path):
    """The cache arrangement the paper proposes: [block][layer][K|V]..."""
    if path == B.KV_PATH_DMA_BLOCKS and layout != B.KV_HOST_BLOCK_FIRST:
        with pytest.raises(B.KVError):          # per-block copies need both sides block-first
            make_case(name, layout, path, **BF)
        return
    case, rot = make_case(name, layout, path, **BF)
    case.rotate(rot)
    case.check()
    case.rotate(rot.inverse())
    case.check()
    case.close()


def test_dma_blocks_merges_runs_and_needs_block_first_cache():
    sh = W.SHAPES["small8b"]
    rng = np.random.default_rng(2)
    # out: blocks 10..41 -> slots 0..31 (one run); in: slots 64..95 -> blocks 100..131 in two runs
    out_ids, out_slots = np.arange(10, 42), np.arange(0, 32)
    in_ids = np.concatenate([np.arange(100, 116), np.arange(200, 216)])
    in_slots = np.arange(64, 96)
    rot = W.Rotation(*(a.astype(np.int32) for a in (out_ids, out_slots, in_ids, in_slots)))
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_DMA_BLOCKS, rot=rot, **BF)
    case.rotate(rot)
    case.check()
    assert case.eng.kv_last_stats()["n_launches"] == 1 + 2
    case.close()
    with pytest.raises(B.KVError):
        make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_DMA_BLOCKS, rot=rot)     # layer-first cache


@pytest.mark.parametrize("hbm_layout", [B.KV_HBM_LAYER_FIRST, B.KV_HBM_BLOCK_FIRST])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("n_out,n_in", [(160, 8), (8, 160), (170, 30), (30, 170), (99, 100), (1, 199), (85, 100)])
def test_unbalanced_rotations(n_out, n_in, layout, hbm_layout):
    """With the in list longer, the kernel spreads the out tiles evenly over the in
    tiles instead of pairing them 1:1; with the out list longer, the rest of it
    follows the paired part (in the same launch, or from 64 MiB on in its own).
    Either way the result is the same rotation."""
    sh = W.KVShape(8, 8, 128, 16, n_hbm_blocks=320, n_host_slots=200)   # 512 KiB blocks
    rot = W.simple_rotation(sh, n_out, n_in, seed=n_out * 1000 + n_in)
    case, _ = make_case(sh, layout, B.KV_PATH_AUTO, rot=rot, hbm_layout=hbm_layout)
    case.rotate(rot)
    case.check()
    # 64 MiB or more of the out list beyond the in list go in a launch of their own
    rest_mib = max(0, n_out - n_in) * 0.5
    assert case.eng.kv_last_stats()["n_launches"] == (2 if rest_mib >= 64 else 1)
    # and back, as one rotation the other way round
    case.rotate(rot.inverse())
    case.check()
    case.close()


@pytest.mark.parametrize("lanes,wgs,u", [(64, 7, 1), (64, 124, 2), (256, 31, 1), (128, 1, 4), (1024, 3, 1)])
def test_in_heavy_interleave_for_every_launch_shape(lanes, wgs, u):
    sh = W.SHAPES["small8b"]
    for n_out, n_in in [(3, 40), (39, 40), (1, 2)]:
        rot = W.simple_rotation(sh, n_out, n_in, seed=n_out * 100 + n_in + lanes)
        case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_FUSED, rot=rot, wg_lanes=lanes, max_copy_wgs=wgs,
                            vecs_per_lane=u)
        case.rotate(rot)
        case.check()
        case.close()


@pytest.mark.parametrize("hbm_layout", [B.KV_HBM_LAYER_FIRST, B.KV_HBM_BLOCK_FIRST])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("u", [0, 2, 4])
def test_in_heavy_interleave_on_ragged_segments(u, layout, hbm_layout):
    """Segments that are not a whole number of tiles (1200 bytes = 75 vectors, tiles
    of 64, 128 or 256): the out tiles spread over a longer in list sit at other
    places of their segments than the in tiles they ride with, so each direction
    needs its own range check."""
    sh = W.SHAPES["ragged"]
    for n_out, n_in in [(1, 12), (5, 12), (6, 12), (2, 3)]:
        rot = W.simple_rotation(sh, n_out, n_in, seed=n_out * 100 + n_in + u)
        case, _ = make_case(sh, layout, B.KV_PATH_FUSED, rot=rot, vecs_per_lane=u, hbm_layout=hbm_layout)
        case.rotate(rot)
        case.check()
        case.rotate(rot.inverse())      # out-heavy: pairs 1:1, the rest alone
        case.check()
        case.close()


def test_racing_calls_are_refused_and_joined_calls_are_not():
    """Un-waited calls run in order per stream and side by side across the two
    streams: a call that would read what un-waited work on the other stream
    writes (or the reverse) gets KV_EBUSY and changes nothing; a launch that
    carries both directions joins the streams, so such rotations may follow one
    another over the same blocks."""
    sh = W.SHAPES["small8b"]
    rot = W.simple_rotation(sh, 12, 10, seed=77)
    inv = rot.inverse()
    # two kernels on two streams: the inverse would read blocks the first call is still writing
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_ZEROCOPY, rot=rot)
    case.rotate(rot)
    assert case.eng.kv_rotate(inv.out_ids, inv.out_slots, inv.in_ids, inv.in_slots) == B.KV_EBUSY
    assert case.eng.kv_swap_out(rot.in_ids[:2], rot.in_slots[:2]) == B.KV_EBUSY      # reads a block being written
    assert case.eng.kv_swap_in(rot.out_slots[:2], rot.in_ids[:2]) == B.KV_EBUSY      # reads a slot being written
    free = np.setdiff1d(np.arange(sh.n_hbm_blocks, dtype=np.int32), np.concatenate([rot.out_ids, rot.in_ids]))
    assert case.eng.kv_swap_in(rot.in_slots[:2], rot.out_ids[:2]) == B.KV_EBUSY      # writes a block being read
    case.check()                                                                     # only the first call happened
    case.rotate(inv)                                                                 # after the wait it is fine
    case.check()
    # same stream, same direction: ordered, so reusing a slot is not a race
    case.swap_out(rot.out_ids[:3], rot.out_slots[:3])
    case.swap_out(rot.out_ids[3:6], rot.out_slots[:3])
    case.swap_out(rot.out_ids[:3], rot.in_slots[:3])
    # the other stream may run beside it on blocks and slots of its own
    case.swap_in(rot.in_slots[3:6], free[:3])
    case.check()
    case.close()
    # one launch for both directions: ordered against everything before and after
    case, _ = make_case(sh, B.KV_HOST_LAYER_FIRST, B.KV_PATH_AUTO, rot=rot)
    case.swap_in(rot.in_slots[:4], free[:4])          # stream_in only ...
    case.rotate(W.Rotation(free[:4], rot.out_slots[:4], rot.in_ids[:4], rot.in_slots[4:8]))   # ... then a join over the same blocks
    case.rotate(rot)
    case.rotate(inv)
    case.rotate(rot)
    case.swap_out(rot.in_ids[:3], rot.out_slots[:3])   # after a join: ordered, although one stream only
    case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY, B.KV_PATH_SDMA_STAGED])
def test_query_polls_without_blocking(path):
    """kv_query: KV_OK with nothing in flight, KV_EBUSY right behind the enqueue of
    128 + 128 MiB (which takes milliseconds), KV_OK some time later without any
    blocking call; the bytes are then in place, and the stats interval is still
    open for kv_wait to close."""
    import time
    sh = W.KVShape(32, 8, 128, 16, n_hbm_blocks=300, n_host_slots=160)       # 2 MiB blocks
    rot = W.simple_rotation(sh, 64, 64, seed=5)
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, path, rot=rot)
    assert case.eng.kv_query() == 0
    assert case.eng.kv_rotate(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots) == 0
    first = case.eng.kv_query()
    deadline, polls = time.time() + 20, 0
    while case.eng.kv_query() == B.KV_EBUSY:
        polls += 1
        assert time.time() < deadline, "the transfer never finished"
        time.sleep(0.0002)
    assert case.eng.kv_query() == 0
    assert first == B.KV_EBUSY and polls > 0, "a transfer of milliseconds was done before the call returned"
    assert O.rotate(case.oshape, case.ref_cache.view(np.uint8), case.ref_pool.view(np.uint8),
                    rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots) == 0
    # in place before any kv_wait: the pool as the CPU sees it, the cache as a copy sees it
    assert np.array_equal(case.pool_u8.view(np.uint16), case.ref_pool)
    assert np.array_equal(case.dev_cache.cpu().numpy().view(np.uint16), case.ref_cache)
    # what would have raced with the finished call is accepted now, without a kv_wait in between
    # (on the two-stream paths the inverse is refused while the first call still runs)
    inv = rot.inverse()
    case.rotate(inv)
    assert case.eng.kv_wait() == 0
    st = case.eng.kv_last_stats()
    assert st["bytes_out"] == st["bytes_in"] == 2 * 64 * (2 << 20)        # one interval: both calls
    assert case.eng.kv_query() == 0
    case.check()
    case.close()
