"""Layer-by-layer transfers of the kernel paths (cfg.chunk_layers > 0): the result
is the oracle's whatever the chunking, and a consumer that waits for layer l only
finds layer l of every block in place while later layers may still be moving."""
import numpy as np
import pytest
import torch

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W
from tests import kvviews as V
from tests.gpu_harness import make_case

pytestmark = pytest.mark.gpu

LAYOUTS = [B.KV_HOST_BLOCK_FIRST, B.KV_HOST_LAYER_FIRST]


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY])
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name,chunk_layers", [("small8b", 1), ("small8b", 3), ("ragged", 2), ("tiny", 1), ("tiny", 5)])
def test_chunked_rotation_matches_oracle(name, chunk_layers, layout, path):
    case, rot = make_case(name, layout, path, chunk_layers=chunk_layers)
    case.rotate(rot)
    case.check()
    n_chunks = -(-case.shape.n_layers // chunk_layers)
    st = case.eng.kv_last_stats()
    # one launch per chunk; the two-kernel path has one per chunk and direction
    assert st["n_launches"] == n_chunks * (2 if path == B.KV_PATH_ZEROCOPY else 1)
    case.rotate(rot.inverse())
    case.check()
    case.swap_out(rot.out_ids[:3], rot.out_slots[:3])       # single directions run layer by layer too
    case.check()
    case.swap_in(rot.out_slots[:2], rot.out_ids[:2])
    case.check()
    # every layer is a valid thing to wait for, outside [0, L) is not
    assert case.eng.kv_wait_layer(0) == 0 and case.eng.kv_wait_layer(case.shape.n_layers - 1) == 0
    assert case.eng.kv_wait_layer(case.shape.n_layers) == B.KV_EINVAL
    assert case.eng.kv_stream_wait_layer(0, -1) == B.KV_EINVAL
    case.close()


@pytest.mark.parametrize("hbm_layout", [B.KV_HBM_LAYER_FIRST, B.KV_HBM_BLOCK_FIRST])
@pytest.mark.parametrize("n_out,n_in", [(40, 6), (6, 40), (24, 30)])
def test_chunked_unbalanced_rotations(n_out, n_in, hbm_layout):
    sh = W.SHAPES["small8b"]
    rot = W.simple_rotation(sh, n_out, n_in, seed=n_out * 10 + n_in)
    case, _ = make_case(sh, B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO, rot=rot, chunk_layers=2, hbm_layout=hbm_layout)
    case.rotate(rot)
    case.check()
    case.rotate(rot.inverse())
    case.check()
    case.close()


@pytest.mark.parametrize("path", [B.KV_PATH_AUTO, B.KV_PATH_ZEROCOPY])
def test_a_consumer_that_waits_for_one_layer_finds_it_complete(path, say):
    """1 GiB each way in 8 chunks of 4 layers.  For every chunk a consumer stream
    waits for the chunk's last layer and then copies those layers of the swapped-in
    blocks aside; all of that is enqueued at once, long before the transfer ends.
    Every copy must hold the bytes that were staged for those layers."""
    sh = W.KVShape(32, 8, 128, 16, n_hbm_blocks=2048, n_host_slots=1100)       # 2 MiB blocks, 4 GiB cache
    n, chunk = 512, 4
    rot = W.simple_rotation(sh, n, n, seed=77)
    dev = torch.empty(V.n_cache_elems(sh), dtype=torch.int16, device="cuda").random_()
    torch.cuda.synchronize()
    eng = B.Engine(B.make_config(sh, path=path, chunk_layers=chunk), dev.data_ptr())
    pool = eng.host_pool_array().view(np.int16).reshape((sh.n_host_slots,) + sh.block_dims())
    staged = np.random.default_rng(3).integers(-32768, 32767, size=(n,) + sh.block_dims(), dtype=np.int16)
    pool[rot.in_slots] = staged
    dv = dev.view(sh.n_layers, 2, sh.n_hbm_blocks, sh.block_size, sh.n_kv_heads, sh.head_dim)
    in_ids = torch.from_numpy(rot.in_ids).long().cuda()
    before_out = dv[:, :, torch.from_numpy(rot.out_ids).long().cuda()].cpu().numpy()
    consumer = torch.cuda.Stream()
    n_chunks = sh.n_layers // chunk
    snaps = [torch.empty((chunk, 2, n, sh.block_size, sh.n_kv_heads, sh.head_dim), dtype=torch.int16, device="cuda")
             for _ in range(n_chunks)]
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_chunks)]
    with torch.cuda.stream(consumer):       # first use of the copy kernel and of the events costs milliseconds: not in the timed part
        torch.index_select(dv[0:chunk], 2, in_ids, out=snaps[0])
        marks[0].record(consumer)
    torch.cuda.synchronize()
    assert eng.kv_rotate(rot.out_ids, rot.out_slots, rot.in_ids, rot.in_slots) == 0
    for c in range(n_chunks):
        assert eng.kv_stream_wait_layer(consumer.cuda_stream, c * chunk + chunk - 1) == 0
        with torch.cuda.stream(consumer):
            torch.index_select(dv[c * chunk:(c + 1) * chunk], 2, in_ids, out=snaps[c])
            marks[c].record(consumer)
    assert eng.kv_wait_layer(0) == 0
    assert eng.kv_wait() == 0
    consumer.synchronize()
    st = eng.kv_last_stats()
    assert st["n_launches"] == n_chunks * (2 if path == B.KV_PATH_ZEROCOPY else 1)
    # the consumer's copies: [chunk layers, 2, n, P, H, D] against staged [n, L, 2, P, H, D]
    for c, snap in enumerate(snaps):
        want = staged[:, c * chunk:(c + 1) * chunk].transpose(1, 2, 0, 3, 4, 5)
        assert np.array_equal(snap.cpu().numpy(), want), f"layers of chunk {c} were not in place when their mark fired"
    # the out direction landed as well
    assert np.array_equal(pool[rot.out_slots].transpose(1, 2, 0, 3, 4, 5), before_out)
    # How far apart the consumer's first and last copy ended: most of the transfer's
    # duration when the consumer's stream has a hardware queue of its own.  Streams share
    # a few hardware queues, so this is reported, not asserted (the rate of the overlap is
    # the business of experiments.py layers).
    spread = marks[0].elapsed_time(marks[-1])
    say(f"consumer's copies spread over {spread:.1f} ms of a {max(st['ms_out'], st['ms_in']):.1f} ms transfer")
    eng.kv_destroy()


def test_unchunked_calls_wait_for_the_whole_call():
    case, rot = make_case("small8b", B.KV_HOST_BLOCK_FIRST, B.KV_PATH_AUTO)     # chunk_layers = 0
    side = torch.cuda.Stream()
    case.rotate(rot)
    assert case.eng.kv_stream_wait_layer(side.cuda_stream, 0) == 0
    with torch.cuda.stream(side):
        snap = case.dev_cache.clone()
    side.synchronize()
    assert np.array_equal(snap.cpu().numpy().view(np.uint16), case.ref_cache)
    assert case.eng.kv_wait_layer(3) == 0
    case.check()
    case.close()


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("staging", [0, 1 << 20])
def test_dma_staged_path_marks_its_layer_chunks(layout, staging):
    """One chunk per layer of the whole list: each chunk gets its mark.  With a staging
    buffer too small for a layer of the whole list (1 MiB) the list is cut and the waits
    fall back to the whole call; either way, what is waited for is in place."""
    case, rot = make_case("small8b", layout, B.KV_PATH_SDMA_STAGED, chunk_layers=1, staging_bytes=staging)
    sh = case.shape
    side = torch.cuda.Stream()
    dv = case.dev_cache.view(sh.n_layers, 2, sh.n_hbm_blocks, sh.block_size, sh.n_kv_heads, sh.head_dim)
    in_ids = torch.from_numpy(rot.in_ids).long().cuda()
    snaps = [torch.empty((1, 2, len(rot.in_ids)) + dv.shape[3:], dtype=torch.int16, device="cuda")
             for _ in range(sh.n_layers)]
    torch.cuda.synchronize()
    case.rotate(rot)
    for l in range(sh.n_layers):
        assert case.eng.kv_stream_wait_layer(side.cuda_stream, l) == 0
        with torch.cuda.stream(side):
            torch.index_select(dv[l:l + 1], 2, in_ids, out=snaps[l])
    assert case.eng.kv_wait_layer(sh.n_layers - 1) == 0
    side.synchronize()
    want = V.hbm_view(sh, case.ref_cache)[:, :, rot.in_ids]
    for l in range(sh.n_layers):
        assert np.array_equal(snaps[l].cpu().numpy().view(np.uint16)[0], want[l]), f"layer {l}"
    case.check()
    case.close()
