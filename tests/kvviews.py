"""Array views of the cache and the host pool, for the tests only.

These are NumPy reshapes of the documented layouts, written independently of
both the oracle's and the library's byte-offset code, so they can serve as a
third opinion on where a segment lives.
"""
import numpy as np

BLOCK_FIRST, LAYER_FIRST = 0, 1


def hbm_view(shape, u16, hbm_layout=0):
    """[L, 2, NB, P, H, D] view of a flat uint16 cache image (0 = layer-first
    [L][2][NB]..., 1 = block-first [NB][L][2]...)."""
    if hbm_layout == 0:
        return u16.reshape(shape.n_layers, 2, shape.n_hbm_blocks, shape.block_size,
                           shape.n_kv_heads, shape.head_dim)
    v = u16.reshape(shape.n_hbm_blocks, shape.n_layers, 2, shape.block_size,
                    shape.n_kv_heads, shape.head_dim)
    return v.transpose(1, 2, 0, 3, 4, 5)


def pool_view(shape, u16, layout):
    """[L, 2, NS, P, H, D] view of a flat uint16 pool image in either layout."""
    if layout == LAYER_FIRST:
        return u16.reshape(shape.n_layers, 2, shape.n_host_slots, shape.block_size,
                           shape.n_kv_heads, shape.head_dim)
    v = u16.reshape(shape.n_host_slots, shape.n_layers, 2, shape.block_size,
                    shape.n_kv_heads, shape.head_dim)
    return v.transpose(1, 2, 0, 3, 4, 5)


def n_cache_elems(shape):
    return int(np.prod(shape.cache_dims()))


def n_pool_elems(shape):
    return int(shape.n_layers * 2 * shape.n_host_slots * shape.block_size *
               shape.n_kv_heads * shape.head_dim)


def make_images(shape, layout, rotation, value_seed, hbm_layout=0):
    """Seeded cache image and pool image (uint16), with the rotation's in_slots
    holding staged N(0,1) blocks and every other slot a recognisable filler."""
    from paper_2601_20309_amd import workloads as W
    import torch
    img = W.cache_image(shape, value_seed).view(torch.int16).numpy().view(np.uint16)   # [L,2,NB,P,H,D]
    cache = np.empty(n_cache_elems(shape), dtype=np.uint16)
    hbm_view(shape, cache, hbm_layout)[...] = img
    pool = np.empty(n_pool_elems(shape), dtype=np.uint16)
    pv = pool_view(shape, pool, layout)
    # filler: slot s holds the 16-bit pattern 0xA000 + s (mod 2^16) so stray writes show
    pv[...] = (0xA000 + np.arange(shape.n_host_slots, dtype=np.uint32) % 0x1000
               ).astype(np.uint16)[None, None, :, None, None, None]
    n_in = len(rotation.in_slots)
    if n_in:
        staged = W.staged_blocks(shape, n_in, value_seed + 50).view(torch.int16).numpy().view(np.uint16)
        # staged is [i][L][2][P][H][D]
        pv[:, :, rotation.in_slots] = staged.transpose(1, 2, 0, 3, 4, 5)
    return cache, pool


def expected_by_indexing(shape, layout, cache, pool, rotation, hbm_layout=0):
    """The rotation written as NumPy array indexing on copies of the images."""
    c2, p2 = cache.copy(), pool.copy()
    cv, pv = hbm_view(shape, c2, hbm_layout), pool_view(shape, p2, layout)
    cv0 = hbm_view(shape, cache, hbm_layout)
    pv0 = pool_view(shape, pool, layout)
    if len(rotation.out_ids):
        pv[:, :, rotation.out_slots] = cv0[:, :, rotation.out_ids]
    if len(rotation.in_ids):
        cv[:, :, rotation.in_ids] = pv0[:, :, rotation.in_slots]
    return c2, p2
