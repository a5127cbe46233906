"""Helpers for the GPU parity tests: seeded global tensors, virtual-rank buffers, conversions.

Placement of a rank's tokens uses the ORACLE's Algorithm-2 map, never the library's, so the
library's own position arithmetic is part of what the comparison checks.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import usp_oracle as orc
from paper_2405_07719_amd import inputs

BF16, FP32 = 0, 1


def to_device(arr: np.ndarray, dtype: int) -> torch.Tensor:
    """Storage array (uint16 bf16 bits, or float32) -> device tensor of the matching torch dtype."""
    if dtype == BF16:
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Device tensor (bf16 or fp32) -> exact float64 NumPy values."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return inputs.from_bf16_bits(t.view(torch.int16).numpy().view(np.uint16)).reshape(t.shape)
    return t.double().numpy()


def gen(seed, tensor_id, bs, positions, heads, hs, dtype):
    """(storage array, exact float64 values) of a seeded N(0,1) tensor [bs, len(positions), len(heads), hs]."""
    if dtype == BF16:
        return inputs.bf16_tensor_at(seed, tensor_id, bs, positions, heads, hs)
    return inputs.fp32_tensor_at(seed, tensor_id, bs, positions, heads, hs)


class Problem:
    """A small USP problem with its global tensors and seq-layout virtual-rank buffers."""

    def __init__(self, seed, bs, L, hc, hk, hs, U, R, causal, zigzag, dtype, with_do=False):
        self.bs, self.L, self.hc, self.hk, self.hs, self.U, self.R = bs, L, hc, hk, hs, U, R
        self.causal, self.zigzag, self.dtype, self.N = causal, zigzag, dtype, U * R
        pos = np.arange(L)
        self.store, self.val = {}, {}
        ids = {"q": (inputs.TENSOR_Q, hc), "k": (inputs.TENSOR_K, hk), "v": (inputs.TENSOR_V, hk)}
        if with_do:
            ids["do"] = (inputs.TENSOR_DO, hc)
        for name, (tid, h) in ids.items():
            self.store[name], self.val[name] = gen(seed, tid, bs, pos, np.arange(h), hs, dtype)

    def rank_positions(self, rank):
        return orc.zigzag_positions(self.L, self.R, self.U, rank // self.U, rank % self.U, self.zigzag)

    def seq_layout(self, name) -> np.ndarray:
        """[N][bs][L/N][heads][hs] storage array: shard of rank r*U+u at its Algorithm-2 positions."""
        g = self.store[name]
        return np.stack([g[:, self.rank_positions(rank)] for rank in range(self.N)])

    def seq_layout_dev(self, name) -> torch.Tensor:
        return to_device(self.seq_layout(name), self.dtype)


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0


def assert_lse_close(got, ref, atol):
    """-inf must match exactly; finite entries within atol."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.array_equal(np.isneginf(got), np.isneginf(ref)), "pattern of -inf LSE entries differs"
    fin = np.isfinite(ref)
    assert np.all(np.isfinite(got[fin]))
    if fin.any():
        err = np.max(np.abs(got[fin] - ref[fin]))
        assert err <= atol, f"LSE max-abs error {err} > {atol}"
