"""Parity at BASELINE's full sizes, in the launch configuration bench.py times
(default config: AUTO path, block-first pool, library-owned pool and streams)."""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests.gpu_harness import BigCase

pytestmark = pytest.mark.gpu


def test_llama3_8b_rotation_full_size():
    """configs[1]: 16 GiB cache, one 2048-token request out while another comes in."""
    case = BigCase("llama3_8b")
    rot = W.config_rotation("llama3_8b")
    assert len(rot.out_ids) == 128 and len(rot.in_ids) == 128
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    st = case.eng.kv_last_stats()
    assert st["path_used"] == B.KV_PATH_FUSED and st["n_launches"] == 1
    assert st["bytes_out"] == st["bytes_in"] == 256 << 20
    case.rotate(rot.inverse())      # what bench.py alternates with
    case.check()
    case.close()


@pytest.mark.parametrize("where", ["named block", "named slot", "other block", "other slot"])
def test_the_full_size_check_notices_one_wrong_byte(where):
    """The check itself: one byte changed on the CPU side (in the oracle's images, or in a
    slot or block that no list names) after a correct rotation makes it fail."""
    case = BigCase("llama3_8b")
    rot = W.config_rotation("llama3_8b")
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    named_b = np.zeros(case.shape.n_hbm_blocks, bool)
    named_b[rot.out_ids] = named_b[rot.in_ids] = True
    named_s = np.zeros(case.shape.n_host_slots, bool)
    named_s[rot.out_slots] = named_s[rot.in_slots] = True
    last_layer = case.shape.n_layers - 1
    if where == "named block":        # the oracle's image of the last block swapped in, last layer, V, last element
        case._cv()[last_layer, 1, rot.in_ids[-1], -1, -1, -1] ^= 1
    elif where == "named slot":
        case._pv(case.ref_pool)[last_layer, 0, rot.out_slots[-1], 0, 0, 0] ^= 0x100
    elif where == "other block":      # a block no list names, changed on the device
        b = int(np.flatnonzero(~named_b)[-1])
        case.cache.view(torch.int16)[last_layer, 1, b, -1, -1, -1] += 1
    else:                             # a slot no list names, changed in the pinned pool
        sl = int(np.flatnonzero(~named_s)[-1])
        case._pv(case.pool_u8)[last_layer, 1, sl, -1, -1, -1] ^= 1
    with pytest.raises(AssertionError):
        case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_SDMA_STAGED, B.KV_PATH_ZEROCOPY])
def test_llama3_8b_rotation_full_size_other_paths(path):
    case = BigCase("llama3_8b", path=path)
    rot = W.config_rotation("llama3_8b", contiguous_slots=True)
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    case.close()


def test_batch_rotation_full_size():
    """configs[2]: 32 requests out and 32 in, lognormal lengths, one call; then
    the same requests as 32 back-to-back calls without waiting."""
    info = W.batch_rotation(W.SHAPES["batch"], W.BASE_SEED + 102)
    rot = info["rotation"]
    assert 1500 < len(rot.out_ids) < 4500 and 1500 < len(rot.in_ids) < 4500
    case = BigCase("batch")
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    # undo (the in list is now the longer one: out tiles spread over the in tiles), then redo
    # request pair by request pair
    case.rotate(rot.inverse())
    case.check()
    bo, bi = info["bounds_out"], info["bounds_in"]
    for r in range(len(bo) - 1):
        case.rotate(W.Rotation(rot.out_ids[bo[r]:bo[r + 1]], rot.out_slots[bo[r]:bo[r + 1]],
                               rot.in_ids[bi[r]:bi[r + 1]], rot.in_slots[bi[r]:bi[r + 1]]))
    case.check()
    case.close()


@pytest.mark.parametrize("path,layout,chunk_layers", [
    (B.KV_PATH_AUTO, B.KV_HOST_BLOCK_FIRST, 0),
    (B.KV_PATH_AUTO, B.KV_HOST_LAYER_FIRST, 1),
    (B.KV_PATH_SDMA_STAGED, B.KV_HOST_LAYER_FIRST, 1),
])
def test_long70b_rotation_full_size(path, layout, chunk_layers, say):
    """configs[3]: 80 layers, 64 KiB segments, 10 MiB blocks, a 45 GiB cache and a
    40 GiB pool; two 32768-token requests leave while two come back (20 GiB each
    way, the transfer size of the paper's Section 5.4 / Table 2 per direction), in
    one launch on the default path, layer by layer on the default path (80 launches,
    each with its completion mark), and chunked per layer on the DMA path."""
    shape = W.SHAPES["long70b"]
    assert shape.n_hbm_blocks == 4608 and shape.n_host_slots == 4096
    rot = W.config_rotation("long70b", contiguous_slots=path == B.KV_PATH_SDMA_STAGED)
    assert len(rot.out_ids) == len(rot.in_ids) == 2048
    case = BigCase("long70b", layout=layout, path=path, chunk_layers=chunk_layers, say=say)
    blk = B.kv_block_bytes(case.cfg)
    assert blk == 10 << 20 and B.kv_cache_bytes(case.cfg) == 45 << 30
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    st = case.eng.kv_last_stats()
    assert st["bytes_out"] == st["bytes_in"] == 20 << 30
    if path == B.KV_PATH_SDMA_STAGED:
        # 80 layer chunks per direction, each one pack / unpack kernel + 2 plane copies
        assert st["path_used"] == B.KV_PATH_SDMA_STAGED and st["n_launches"] == 2 * 80 * 3
    else:
        assert st["path_used"] == B.KV_PATH_FUSED and st["n_launches"] == (80 if chunk_layers == 1 else 1)
        assert case.eng.kv_wait_layer(79) == 0
    case.close()


def test_interference_rotation_beside_the_reader_full_size(say):
    """configs[4]: Llama-3-8B shape, 48 GiB cache; eight 4096-token requests leave
    while eight come back (2048 + 2048 blocks, 4 GiB each way) and the decode
    reader streams 19200 other blocks (37.5 GiB per pass) at the same time.  Cache,
    pool and the reader's checksum are all checked against the oracle."""
    shape = W.SHAPES["interference"]
    assert shape.n_hbm_blocks == 24576
    rot = W.config_rotation("interference")
    assert len(rot.out_ids) == len(rot.in_ids) == 2048
    named = np.zeros(shape.n_hbm_blocks, dtype=bool)
    named[rot.out_ids] = named[rot.in_ids] = True
    others = np.flatnonzero(~named)
    read_ids = np.random.default_rng(W.BASE_SEED + 204).permutation(others)[:19200].astype(np.int32)
    case = BigCase("interference", say=say)
    case.stage(rot.in_slots)
    case.sync_ref(read_ids, read_only=True)
    rc, want = O.read_checksum(case.oshape, case.ref_cache, read_ids)
    assert rc == 0
    say("oracle checksum of the reader's blocks done")
    passes = 16                           # ~110 ms of reading; the rotation needs ~85 ms
    case.sync_ref(np.concatenate([rot.out_ids, rot.in_ids]), np.concatenate([rot.out_slots, rot.in_slots]))
    assert case.eng.kv_reader_start(read_ids, passes) == 0
    case.rotate(rot)                      # enqueued while the reader runs
    rc, got, ms = case.eng.kv_reader_wait()
    assert rc == 0 and len(ms) == passes and got == (want * passes) % (1 << 64)
    case.check()
    st = case.eng.kv_last_stats()
    assert st["path_used"] == B.KV_PATH_FUSED and st["bytes_out"] == st["bytes_in"] == 4 << 30
    say(f"rotation {st['ms_out']:.1f} ms beside a reader of {sum(ms):.1f} ms in {passes} passes")
    # and the inverse, with the reader over the same blocks once more
    assert case.eng.kv_reader_start(read_ids, 1) == 0
    case.rotate(rot.inverse())
    rc, got, _ = case.eng.kv_reader_wait()
    assert rc == 0 and got == want
    case.check()
    case.close()
