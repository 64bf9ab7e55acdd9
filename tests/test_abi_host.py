"""CPU-side checks of the HIP library: it loads, exports what the header
declares, and its host logic (sizes, admission) agrees with the oracle.
No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import kv_oracle as O
from paper_2601_20309_amd import binding as B
from paper_2601_20309_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "duplexkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(kv_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_codes_match_header_and_oracle():
    text = open(os.path.join(ROOT, "include", "duplexkv.h")).read()
    codes = {k: int(v) for k, v in re.findall(r"#define\s+(KV_E?[A-Z0-9]+)\s+\(?(-?\d+)\)?", text)}
    for name in ("KV_OK", "KV_EINVAL", "KV_ERANGE", "KV_EDUP", "KV_EOVERLAP", "KV_ENOMEM",
                 "KV_EHIP", "KV_EUNSUP", "KV_ENOSPC", "KV_EBUSY", "KV_E2BIG"):
        assert codes[name] == getattr(B, name)
    assert (B.KV_OK, B.KV_EINVAL, B.KV_ERANGE, B.KV_EDUP, B.KV_EOVERLAP, B.KV_ENOSPC) == \
           (O.OK, O.EINVAL, O.ERANGE, O.EDUP, O.EOVERLAP, O.ENOSPC)
    states = {k: int(v) for k, v in re.findall(r"#define\s+(KV_BLOCK_[A-Z]+)\s+(\d+)", text)}
    assert (states["KV_BLOCK_DIRTY"], states["KV_BLOCK_FULL"], states["KV_BLOCK_SYNCED"], states["KV_BLOCK_HOST"]) == \
           (O.DIRTY, O.FULL, O.SYNCED, O.HOST) == (B.KV_BLOCK_DIRTY, B.KV_BLOCK_FULL, B.KV_BLOCK_SYNCED, B.KV_BLOCK_HOST)
    for c in range(-10, 1):
        assert B.kv_strerror(c) != "unknown code"
    assert B.kv_strerror(-99) == "unknown code"


@pytest.mark.parametrize("name", sorted(W.SHAPES))
def test_sizes_agree_with_oracle(name):
    sh = W.SHAPES[name]
    for layout in (0, 1):
        cfg, s = B.make_config(sh, layout), O.shape_of(sh, layout)
        assert B.kv_seg_bytes(cfg) == O.seg_bytes(s)
        assert B.kv_block_bytes(cfg) == O.block_bytes(s)
        assert B.kv_cache_bytes(cfg) == O.cache_bytes(s)
        assert B.kv_pool_bytes(cfg) == O.pool_bytes(s)


def test_bad_config_sizes_are_zero_and_validate_rejects():
    sh = W.SHAPES["tiny"]
    for field, val in [("n_layers", 0), ("host_layout", 2), ("path", 9), ("vecs_per_lane", 3), ("hbm_layout", 2), ("path", 6), ("wg_lanes", 100), ("wg_lanes", 2048),
                       ("elem_bytes", -2), ("chunk_layers", -1)]:
        cfg = B.make_config(sh)
        setattr(cfg, field, val)
        assert B.kv_cache_bytes(cfg) == 0
        assert B.kv_validate(cfg, [1], [1], None, None) == B.KV_EINVAL


def test_validate_agrees_with_oracle_on_random_lists():
    sh = W.KVShape(1, 1, 8, 2, n_hbm_blocks=9, n_host_slots=7)
    cfg, s = B.make_config(sh), O.shape_of(sh)
    rng = np.random.default_rng(99)
    seen = set()
    for _ in range(5000):
        no, ni = rng.integers(0, 4, size=2)
        oi = rng.integers(-1, sh.n_hbm_blocks + 1, size=no)
        os_ = rng.integers(-1, sh.n_host_slots + 1, size=no)
        ii = rng.integers(-1, sh.n_hbm_blocks + 1, size=ni)
        is_ = rng.integers(-1, sh.n_host_slots + 1, size=ni)
        want = O.validate(s, oi, os_, ii, is_)
        assert B.kv_validate(cfg, oi, os_, ii, is_) == want
        seen.add(want)
    assert seen == {0, -2, -3, -4}


def test_validate_large_lists_and_einval():
    sh = W.SHAPES["llama3_8b"]
    cfg, s = B.make_config(sh), O.shape_of(sh)
    rng = np.random.default_rng(5)
    perm = rng.permutation(sh.n_hbm_blocks).astype(np.int32)
    sperm = rng.permutation(sh.n_host_slots).astype(np.int32)
    n = sh.n_host_slots // 2
    args = (perm[:n], sperm[:n], perm[n:2 * n], sperm[n:2 * n])
    assert B.kv_validate(cfg, *args) == 0 == O.validate(s, *args)
    bad = (perm[:n], sperm[:n], perm[n - 1:2 * n - 1], sperm[n:2 * n])   # one shared block
    assert B.kv_validate(cfg, *bad) == B.KV_EOVERLAP == O.validate(s, *bad)
    assert B.kv_validate(cfg, None, None, None, None) == 0
    assert B.kv_validate(cfg, None, None, None, None, n_out=3) == B.KV_EINVAL
    assert B.kv_validate(cfg, None, None, None, None, n_in=-1) == B.KV_EINVAL


def test_create_fails_loudly_without_gpu_or_with_bad_arguments():
    import torch
    cfg = B.make_config(W.SHAPES["tiny"])
    handle = ctypes.c_void_p()
    assert B.lib.kv_create(None, ctypes.byref(cfg), None, None, None, None) == B.KV_EINVAL
    assert B.lib.kv_create(ctypes.byref(handle), ctypes.byref(cfg), None, None, None, None) == B.KV_EINVAL
    if not torch.cuda.is_available():
        with pytest.raises(B.KVError) as ei:
            B.Engine(cfg, 0x10000)
        assert ei.value.code == B.KV_EHIP
    assert B.lib.kv_wait(None) == B.KV_EINVAL
    assert B.lib.kv_rotate(None, None, None, 0, None, None, 0) == B.KV_EINVAL
    assert B.lib.kv_destroy(None) == B.KV_EINVAL
    assert B.lib.kv_table_create(ctypes.byref(handle), None, 4) == B.KV_EINVAL
    assert B.lib.kv_table_rotate(None, None, 0, None, 0) == B.KV_EINVAL
    assert B.lib.kv_table_destroy(None) == B.KV_EINVAL
