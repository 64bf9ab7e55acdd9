"""Parity at BASELINE's full sizes, in the launch configuration bench.py times
(default config: AUTO path, block-first pool, library-owned pool and streams)."""
import dataclasses

import numpy as np
import pytest

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
    (B.KV_PATH_SDMA_STAGED, B.KV_HOST_LAYER_FIRST, 1),
])
def test_long70b_shape_quarter_size(path, layout, chunk_layers):
    """configs[3] shape (80 layers, 64 KiB segments, 10 MiB blocks) at a quarter of
    its block counts: 2 x 8192-token requests each way, chunked per layer on the
    DMA path.  The full-size run is bench.py --workload long70b."""
    shape = dataclasses.replace(W.SHAPES["long70b"], n_hbm_blocks=1152, n_host_slots=1024)
    rot = W.request_rotation(shape, [8192] * 2, [8192] * 2, seed=W.BASE_SEED + 103, contiguous_slots=True)
    assert len(rot.out_ids) == 512
    case = BigCase("long70b", layout=layout, path=path, shape=shape, chunk_layers=chunk_layers)
    case.stage(rot.in_slots)
    case.rotate(rot)
    case.check()
    if chunk_layers == 1:
        # 80 layer chunks per direction, each one pack/unpack kernel + 2 plane copies
        assert case.eng.kv_last_stats()["n_launches"] == 2 * 80 * 3
    case.close()
