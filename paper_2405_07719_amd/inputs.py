"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds data generation only: a counter-based pseudo-random generator
keyed on (seed, tensor id, batch, global position, head, element), a Box-Muller
transform to N(0,1), and the bf16 storage conversion.  It contains none of the
attention / layout / merge arithmetic, so both the CPU oracle's tests and the HIP
path can be fed from it without sharing any of the method's code.

Because the value of an element depends only on its global coordinates, any
virtual rank's shard can be materialised without building the global tensor.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_DO = 0, 1, 2, 3

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        x = ((x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        x = ((x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        x = x ^ (x >> np.uint64(31))
    return x


def normal_at(seed: int, tensor_id: int, b, pos, head, elem) -> np.ndarray:
    """N(0,1) value (float64) at the given coordinates; arguments broadcast.

    The counter is a 64-bit mix of the coordinates, so the value at a coordinate
    never depends on which other coordinates are requested.
    """
    b = np.asarray(b, dtype=np.uint64)
    pos = np.asarray(pos, dtype=np.uint64)
    head = np.asarray(head, dtype=np.uint64)
    elem = np.asarray(elem, dtype=np.uint64)
    with np.errstate(over="ignore"):
        key = _splitmix64(np.uint64(seed) * np.uint64(0x100000001B3) + np.uint64(tensor_id + 1))
        ctr = ((b * np.uint64(1 << 24) + head) * np.uint64(1 << 12) + elem) * np.uint64(1 << 26) + pos
        bits = _splitmix64(ctr ^ key)
    hi = (bits >> np.uint64(40)).astype(np.float64)            # 24 bits
    lo = ((bits >> np.uint64(8)) & np.uint64(0xFFFFFF)).astype(np.float64)
    u1 = (hi + 1.0) / 16777216.0                                 # (0, 1]
    u2 = lo / 16777216.0                                         # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def tensor_at(seed: int, tensor_id: int, bs: int, positions, heads, hs: int, dtype=np.float64,
              threads: int = 8) -> np.ndarray:
    """float64 (or `dtype`) array [bs, len(positions), len(heads), hs] of N(0,1) values.

    `positions` are global sequence positions and `heads` global head indices,
    so a shard of any virtual rank is `tensor_at(..., its positions, its heads)`.
    """
    positions = np.asarray(positions, dtype=np.uint64)
    heads = np.asarray(heads, dtype=np.uint64)
    out = np.empty((bs, positions.size, heads.size, hs), dtype=dtype)
    e = np.arange(hs, dtype=np.uint64)[None, None, :]
    step = max(1, (1 << 20) // max(1, heads.size * hs))

    def fill(job):
        b, s = job
        p = positions[s:s + step, None, None]
        out[b, s:s + step] = normal_at(seed, tensor_id, b, p, heads[None, :, None], e)

    jobs = [(b, s) for b in range(bs) for s in range(0, positions.size, step)]
    if len(jobs) > 1 and threads > 1:
        # NumPy releases the GIL inside its loops; chunks are independent by construction
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64/float32 values to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def bf16_tensor_at(seed, tensor_id, bs, positions, heads, hs):
    """(bits uint16, exact float64 values of those bits) for a bf16 input tensor."""
    bits = to_bf16_bits(tensor_at(seed, tensor_id, bs, positions, heads, hs))
    return bits, from_bf16_bits(bits)


def fp32_tensor_at(seed, tensor_id, bs, positions, heads, hs):
    """(float32 array, its exact float64 widening) for an fp32 input tensor."""
    f = tensor_at(seed, tensor_id, bs, positions, heads, hs).astype(np.float32)
    return f, f.astype(np.float64)
