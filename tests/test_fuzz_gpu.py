"""Random small cases through the C ABI against the oracle: shapes that are
powers of two nowhere, every path, layout, chunking and launch-shape knob in
random combination, lists from empty to nearly everything, two or three calls per
case.  Whole cache and whole pool are compared after every case."""
import numpy as np
import pytest

from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V
from tests.gpu_harness import GpuCase

pytestmark = pytest.mark.gpu


def random_case(rng):
    elem = int(rng.choice([1, 2, 2, 2, 4]))
    sh = W.KVShape(int(rng.integers(1, 6)), int(rng.integers(1, 4)), int(rng.choice([4, 8, 20, 40, 64, 96])),
                   int(rng.integers(1, 8)), n_hbm_blocks=int(rng.integers(6, 40)), n_host_slots=int(rng.integers(6, 40)),
                   elem_bytes=elem)
    if elem == 1 and (sh.block_size * sh.n_kv_heads * sh.head_dim) % 2:
        sh = W.KVShape(sh.n_layers, sh.n_kv_heads, sh.head_dim, sh.block_size + 1, sh.n_hbm_blocks, sh.n_host_slots, elem)
    layout = int(rng.choice([B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST]))
    hbm_layout = int(rng.choice([B.KV_HBM_LAYER_FIRST, B.KV_HBM_BLOCK_FIRST]))
    paths = [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY, B.KV_PATH_FUSED, B.KV_PATH_SDMA_STAGED, B.KV_PATH_NAIVE]
    if layout == B.KV_HOST_BLOCK_FIRST and hbm_layout == B.KV_HBM_BLOCK_FIRST:
        paths.append(B.KV_PATH_DMA_BLOCKS)
    path = int(rng.choice(paths))
    kw = dict(hbm_layout=hbm_layout, chunk_layers=int(rng.choice([0, 0, 1, 2, 3])))
    if rng.random() < 0.4:
        kw["max_copy_wgs"] = int(rng.choice([1, 2, 5, 33]))
    if rng.random() < 0.4:
        kw["vecs_per_lane"] = int(rng.choice([1, 2, 4, 8]))
    if rng.random() < 0.3:
        kw["wg_lanes"] = int(rng.choice([64, 128, 320]))
    if path == B.KV_PATH_SDMA_STAGED and rng.random() < 0.5:
        seg = sh.block_size * sh.n_kv_heads * sh.head_dim * sh.elem_bytes
        kw["staging_bytes"] = int(max(2 * seg, 256) * rng.integers(1, 9) + 256)
    return sh, layout, path, kw


def elems16(sh, n_blocks):
    return sh.n_layers * 2 * n_blocks * sh.block_size * sh.n_kv_heads * sh.head_dim * sh.elem_bytes // 2


@pytest.mark.parametrize("seed", range(16))
def test_random_cases_match_the_oracle(seed):
    rng = np.random.default_rng(7000 + seed)
    ran = moved = 0
    for k in range(60):
        sh, layout, path, kw = random_case(rng)
        cache = rng.integers(0, 65536, elems16(sh, sh.n_hbm_blocks), dtype=np.uint16)
        pool = rng.integers(0, 65536, elems16(sh, sh.n_host_slots), dtype=np.uint16)
        try:
            case = GpuCase(sh, layout, path, cache, pool, **kw)
        except B.KVError as ex:
            # the only configuration a random draw may legitimately hit: staging smaller than two segments
            assert ex.code == B.KV_EINVAL and path == B.KV_PATH_SDMA_STAGED, (seed, k, sh, path, kw)
            continue
        what = f"seed {seed} case {k}: {sh}, layout {layout}, path {path}, {kw}"
        for step in range(int(rng.integers(1, 4))):
            cap = min(sh.n_hbm_blocks, sh.n_host_slots)
            n_out = int(rng.integers(0, cap // 2 + 1))
            n_in = int(rng.integers(0, cap - n_out - (cap // 4) + 1))
            ids = rng.permutation(sh.n_hbm_blocks)[:n_out + n_in].astype(np.int32)
            slots = rng.permutation(sh.n_host_slots)[:n_out + n_in].astype(np.int32)
            rot = W.Rotation(ids[:n_out], slots[:n_out], ids[n_out:], slots[n_out:])
            try:
                case.rotate(rot)
                case.check()            # waits, then compares every byte
                moved += n_out + n_in
            except AssertionError as ex:
                raise AssertionError(f"{what}, step {step}, {n_out} out / {n_in} in: {ex}") from ex
        case.close()
        ran += 1
    assert ran >= 50 and moved > 300, (ran, moved)
