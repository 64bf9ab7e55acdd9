"""Seeded synthetic inputs for the KV rotation path.

This module only draws inputs: cache shapes, bf16 fills and block / slot id
lists.  It holds none of the rotation's own arithmetic (no byte offsets, no
copying, no validation), so the CPU oracle and the HIP path can both be fed
from it without sharing any of the method.

The paper measured on KV caches of LLaMA-3-8B, Qwen2.5-32B and Mixtral-8x7B
under ShareGPT / LMSYS-Chat-1M traffic (Section 5.1).  A byte mover only sees
the cache *shape* and the request-length mix, so the stand-ins here are
bf16 ~ N(0,1) tensors of those shapes and seeded random block placements.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch

BASE_SEED = 203090  # 20309 * 10; + config index for values, + 100 for ids


@dataclasses.dataclass(frozen=True)
class KVShape:
    """Shape of a paged KV cache [layer][K|V][block][block_size][kv_heads][head_dim]."""

    n_layers: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    n_hbm_blocks: int
    n_host_slots: int
    elem_bytes: int = 2  # bf16

    def cache_dims(self):
        return (self.n_layers, 2, self.n_hbm_blocks, self.block_size,
                self.n_kv_heads, self.head_dim)

    def block_dims(self):
        """Dims of one block across every layer and both planes."""
        return (self.n_layers, 2, self.block_size, self.n_kv_heads, self.head_dim)


@dataclasses.dataclass
class Rotation:
    """One duplex rotation request: blocks leaving HBM and blocks coming back."""

    out_ids: np.ndarray    # HBM block ids to move out
    out_slots: np.ndarray  # host slots that receive them
    in_ids: np.ndarray     # HBM block ids (free) that receive staged blocks
    in_slots: np.ndarray   # host slots that hold the staged blocks

    def inverse(self) -> "Rotation":
        """The rotation that undoes this one (state returns after both)."""
        return Rotation(self.in_ids.copy(), self.in_slots.copy(),
                        self.out_ids.copy(), self.out_slots.copy())


SHAPES: Dict[str, KVShape] = {
    # configs[0]
    "tiny": KVShape(2, 2, 64, 16, n_hbm_blocks=64, n_host_slots=32),
    # a ragged shape that is not a power of two anywhere (parity edge case)
    "ragged": KVShape(3, 3, 40, 5, n_hbm_blocks=37, n_host_slots=19),
    # mid-size: several tiles per segment, still seconds for the oracle
    "small8b": KVShape(4, 8, 128, 16, n_hbm_blocks=256, n_host_slots=128),
    # configs[1]: Llama-3-8B-shaped KV
    "llama3_8b": KVShape(32, 8, 128, 16, n_hbm_blocks=8192, n_host_slots=2048),
    # configs[2]: batch rotation, same model shape, larger host pool
    "batch": KVShape(32, 8, 128, 16, n_hbm_blocks=8192, n_host_slots=8192),
    # configs[3]: 70B-shaped long context
    "long70b": KVShape(80, 8, 128, 32, n_hbm_blocks=4608, n_host_slots=4096),
    # configs[4]: interference, Llama-3-8B shape with room for the decode reader
    "interference": KVShape(32, 8, 128, 16, n_hbm_blocks=24576, n_host_slots=4096),
    # the paper's Table 2 workload shape (Qwen2.5-32B: 64 layers, 8 KV heads x 128)
    "qwen25_32b": KVShape(64, 8, 128, 16, n_hbm_blocks=4608, n_host_slots=4096),
}


def _gen(seed: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal_bf16(dims, seed: int, device: str = "cpu") -> torch.Tensor:
    """bf16 tensor ~ N(0,1), drawn in fp32 and rounded to nearest-even.

    The stream differs between devices (torch uses different generators on CPU
    and GPU); either is a valid seeded draw.  Whoever consumes the tensor on the
    other side copies these exact bytes, nothing is drawn twice.
    """
    g = _gen(seed, device)
    dims = tuple(int(d) for d in dims)
    out = torch.empty(dims, dtype=torch.bfloat16, device=device)
    # one leading-axis slice at a time keeps the fp32 temporary small
    for i in range(dims[0]):
        out[i] = torch.randn(dims[1:], generator=g, dtype=torch.float32,
                             device=device).to(torch.bfloat16)
    return out


def raw_bits_bf16(dims, seed: int, device: str = "cpu") -> torch.Tensor:
    """bf16 tensor whose 16-bit patterns are uniform random: NaN payloads,
    infinities, signed zeros and subnormals all occur."""
    g = _gen(seed, device)
    bits = torch.randint(-32768, 32768, tuple(int(d) for d in dims), generator=g,
                         dtype=torch.int16, device=device)
    return bits.view(torch.bfloat16)


def cache_image(shape: KVShape, seed: int, device: str = "cpu",
                n_raw_blocks: int = 2) -> torch.Tensor:
    """The whole HBM cache: N(0,1) bf16 with a few blocks of raw random bits."""
    img = normal_bf16(shape.cache_dims(), seed, device)
    rng = np.random.default_rng(seed + 7)
    for k, b in enumerate(rng.choice(shape.n_hbm_blocks,
                                     size=min(n_raw_blocks, shape.n_hbm_blocks),
                                     replace=False)):
        img[:, :, int(b)] = raw_bits_bf16(shape.block_dims(), seed + 11 + k, device)
    return img


def staged_blocks(shape: KVShape, n: int, seed: int, device: str = "cpu") -> torch.Tensor:
    """n blocks worth of staged KV, indexed [i][layer][K|V][t][h][d].

    Which host slot block i sits in, and how the pool lays it out, is the
    method's business; the caller places these through the pool's own view.
    """
    if n == 0:
        return torch.empty((0,) + shape.block_dims(), dtype=torch.bfloat16, device=device)
    return normal_bf16((n,) + shape.block_dims(), seed, device)


def blocks_for_tokens(tokens: int, block_size: int) -> int:
    return (int(tokens) + block_size - 1) // block_size


def lognormal_lengths(n: int, seed: int, median: float = 1024.0, sigma: float = 0.8,
                      lo: int = 64, hi: int = 8192) -> np.ndarray:
    """Request lengths in tokens: lognormal around `median`, clipped to [lo, hi]."""
    rng = np.random.default_rng(seed)
    x = rng.lognormal(mean=math.log(median), sigma=sigma, size=n)
    return np.clip(np.rint(x), lo, hi).astype(np.int64)


def simple_rotation(shape: KVShape, n_out: int, n_in: int, seed: int,
                    n_used: Optional[int] = None,
                    contiguous_slots: bool = False) -> Rotation:
    """n_out random used blocks leave, n_in staged blocks land in random free ids.

    Blocks [perm[:n_used]] count as used, the rest as free; out ids come from the
    used set, in ids from the free set, slots from disjoint parts of one slot
    permutation (or two consecutive runs when `contiguous_slots`).
    """
    rng = np.random.default_rng(seed)
    nb, ns = shape.n_hbm_blocks, shape.n_host_slots
    if n_used is None:
        n_used = nb - max(n_in, (nb - n_out) // 2)
    assert n_out <= n_used and n_in <= nb - n_used and n_out + n_in <= ns
    perm = rng.permutation(nb)
    used, free = perm[:n_used], perm[n_used:]
    out_ids = rng.choice(used, size=n_out, replace=False)
    in_ids = rng.choice(free, size=n_in, replace=False)
    if contiguous_slots:
        start_in = int(rng.integers(0, ns - n_out - n_in + 1))
        in_slots = np.arange(start_in, start_in + n_in)
        out_slots = np.arange(start_in + n_in, start_in + n_in + n_out)
    else:
        sperm = rng.permutation(ns)
        in_slots, out_slots = sperm[:n_in], sperm[n_in:n_in + n_out]
    as32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    return Rotation(as32(out_ids), as32(out_slots), as32(in_ids), as32(in_slots))


def batch_rotation(shape: KVShape, seed: int, n_requests: int = 64,
                   lengths: Optional[np.ndarray] = None) -> Dict[str, object]:
    """configs[2]: half the requests are resident and rotate out, half are staged
    and rotate in; block ids are one global random permutation dealt in order."""
    nb, ns = shape.n_hbm_blocks, shape.n_host_slots
    for attempt in range(64):
        lens = lengths if lengths is not None else lognormal_lengths(n_requests, seed + attempt)
        nblk = np.array([blocks_for_tokens(t, shape.block_size) for t in lens])
        half = n_requests // 2
        tot_out, tot_in = int(nblk[:half].sum()), int(nblk[half:].sum())
        if tot_out + tot_in <= nb and tot_out + tot_in <= ns:
            break
        assert lengths is None, "given lengths do not fit"
    else:
        raise RuntimeError("no draw fits the cache")
    rng = np.random.default_rng(seed + 1000)
    perm = rng.permutation(nb)
    sperm = rng.permutation(ns)
    out_ids, in_ids = perm[:tot_out], perm[tot_out:tot_out + tot_in]
    in_slots, out_slots = sperm[:tot_in], sperm[tot_in:tot_in + tot_out]
    as32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    rot = Rotation(as32(out_ids), as32(out_slots), as32(in_ids), as32(in_slots))
    bounds_out = np.concatenate([[0], np.cumsum(nblk[:half])]).astype(np.int64)
    bounds_in = np.concatenate([[0], np.cumsum(nblk[half:])]).astype(np.int64)
    return {"rotation": rot, "lengths": lens, "bounds_out": bounds_out,
            "bounds_in": bounds_in}


def request_rotation(shape: KVShape, tokens_out: List[int], tokens_in: List[int],
                     seed: int, contiguous_slots: bool = False) -> Rotation:
    """Whole requests of the given token lengths rotate out / in."""
    n_out = sum(blocks_for_tokens(t, shape.block_size) for t in tokens_out)
    n_in = sum(blocks_for_tokens(t, shape.block_size) for t in tokens_in)
    return simple_rotation(shape, n_out, n_in, seed, contiguous_slots=contiguous_slots)


def config_rotation(name: str, contiguous_slots: bool = False) -> Rotation:
    """The rotation each BASELINE config names, with its fixed seed."""
    shape = SHAPES[name]
    idx = {"tiny": 0, "llama3_8b": 1, "batch": 2, "long70b": 3, "interference": 4,
           "qwen25_32b": 5, "ragged": 6, "small8b": 7}[name]
    seed = BASE_SEED + 100 + idx
    if name == "tiny":
        return simple_rotation(shape, 8, 8, seed, n_used=40)
    if name == "ragged":
        return simple_rotation(shape, 7, 5, seed)
    if name == "small8b":
        return simple_rotation(shape, 48, 40, seed)
    if name == "llama3_8b":
        return request_rotation(shape, [2048], [2048], seed, contiguous_slots)
    if name == "batch":
        return batch_rotation(shape, seed)["rotation"]
    if name == "long70b":
        return request_rotation(shape, [32768] * 2, [32768] * 2, seed, contiguous_slots)
    if name == "interference":
        return request_rotation(shape, [4096] * 8, [4096] * 8, seed, contiguous_slots)
    if name == "qwen25_32b":
        return request_rotation(shape, [32768], [32768], seed, contiguous_slots)
    raise KeyError(name)


def value_seed(name: str) -> int:
    idx = {"tiny": 0, "llama3_8b": 1, "batch": 2, "long70b": 3, "interference": 4,
           "qwen25_32b": 5, "ragged": 6, "small8b": 7}[name]
    return BASE_SEED + idx
