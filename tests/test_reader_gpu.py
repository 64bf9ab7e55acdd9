"""The synthetic decode reader against the oracle's checksum, alone and while a
rotation runs."""
import numpy as np
import pytest

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests.gpu_harness import make_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny", "ragged", "small8b"])
def test_reader_checksum_matches_oracle(name):
    case, rot = make_case(name, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO)
    sh = case.shape
    rng = np.random.default_rng(1)
    for ids, passes, wgs in [(rng.permutation(sh.n_hbm_blocks)[: sh.n_hbm_blocks // 2], 1, 0),
                             (np.arange(sh.n_hbm_blocks), 3, 0),
                             (np.array([5, 5, 7]), 2, 3),
                             (np.array([], dtype=np.int32), 1, 0)]:
        rc, want = O.read_checksum(case.oshape, case.ref_cache.view(np.uint8), ids)
        assert rc == 0
        assert case.eng.kv_reader_start(ids, passes, wgs) == 0
        rc, got, ms = case.eng.kv_reader_wait()
        assert rc == 0 and len(ms) == passes
        assert got == (want * passes) % (1 << 64)
    assert case.eng.kv_reader_start([sh.n_hbm_blocks], 1) == B.KV_ERANGE
    assert case.eng.kv_reader_start([0], 0) == B.KV_EINVAL
    assert case.eng.kv_reader_wait()[0] == B.KV_EINVAL     # nothing started
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_SDMA_STAGED])
def test_reader_runs_beside_a_rotation(path):
    """Reader over blocks the rotation does not name, started first, rotation on
    top of it: both results must be what each gives alone."""
    case, rot = make_case("small8b", B.KV_HOST_BLOCK_FIRST, path)
    named = set(rot.out_ids.tolist()) | set(rot.in_ids.tolist())
    others = np.array([b for b in range(case.shape.n_hbm_blocks) if b not in named], dtype=np.int32)
    rc, want = O.read_checksum(case.oshape, case.ref_cache.view(np.uint8), others)
    assert case.eng.kv_reader_start(others, 8) == 0
    case.rotate(rot)
    rc, got, ms = case.eng.kv_reader_wait()
    assert rc == 0 and got == (want * 8) % (1 << 64)
    case.check()
    # swapped-out blocks are only read by the rotation: a reader may share them
    assert case.eng.kv_reader_start(rot.out_ids, 2) == 0
    case.rotate(rot.inverse())
    rc, want2 = O.read_checksum(case.oshape, case.ref_cache.view(np.uint8), rot.out_ids)
    # (the inverse rotation rewrites out_ids with their own bytes, so the sum is stable)
    rc, got2, _ = case.eng.kv_reader_wait()
    assert got2 == (want2 * 2) % (1 << 64)
    case.check()
    case.close()


def test_reader_on_block_first_cache():
    case, rot = make_case("small8b", B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO, hbm_layout=B.KV_HBM_BLOCK_FIRST)
    ids = np.random.default_rng(4).permutation(case.shape.n_hbm_blocks)[:100]
    rc, want = O.read_checksum(case.oshape, case.ref_cache.view(np.uint8), ids)
    assert case.eng.kv_reader_start(ids, 2) == 0
    rc, got, _ = case.eng.kv_reader_wait()
    assert rc == 0 and got == (2 * want) % (1 << 64)
    case.close()
