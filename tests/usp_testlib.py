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


class OneRankCase:
    """A full-size problem of which only ONE virtual rank is run: seq-layout device buffers are allocated at
    full size but only the slices that rank reads are filled (the rest stays zero and is never touched)."""

    def __init__(self, usp, seed, bs, L, hc, hk, hs, U, R, rank, zigzag=True, with_do=False):
        self.usp, self.seed = usp, seed
        self.bs, self.L, self.hc, self.hk, self.hs, self.U, self.R, self.rank = bs, L, hc, hk, hs, U, R, rank
        self.N, self.zigzag = U * R, zigzag
        self.r, self.u = divmod(rank, U)
        self.hq, self.hkv, self.Lq, self.n = hc // U, hk // U, L // R, L // (U * R)
        self.q_heads = np.arange(self.u * self.hq, (self.u + 1) * self.hq)
        self.kv_heads = np.arange(self.u * self.hkv, (self.u + 1) * self.hkv)
        self.p = usp.problem(bs, L, hc, hk, hs, U, R, True, usp.USP_SPLIT_ZIGZAG if zigzag else usp.USP_SPLIT_CONTIG,
                             usp.USP_BF16)
        # Q (and dO): the U shards of ring row r, this rank's head slice.  K, V: all N shards, its KV head slice.
        row_ranks = [self.r * U + up for up in range(U)]
        self.q = self._buffer(inputs.TENSOR_Q, hc, self.q_heads, row_ranks)
        self.k = self._buffer(inputs.TENSOR_K, hk, self.kv_heads, range(self.N))
        self.v = self._buffer(inputs.TENSOR_V, hk, self.kv_heads, range(self.N))
        self.d_o = self._buffer(inputs.TENSOR_DO, hc, self.q_heads, row_ranks) if with_do else None
        self.block_pos = orc.ring_block_positions(L, R, self.r, zigzag)      # positions of the rank's Lq local rows

    def shard_positions(self, rk):
        return orc.zigzag_positions(self.L, self.R, self.U, rk // self.U, rk % self.U, self.zigzag)

    def _buffer(self, tensor_id, heads, read_heads, ranks):
        buf = torch.zeros((self.N, self.bs, self.n, heads, self.hs), dtype=torch.bfloat16, device="cuda")
        for rk in ranks:
            bits = inputs.to_bf16_bits(inputs.tensor_at(self.seed, tensor_id, self.bs, self.shard_positions(rk), read_heads,
                                                        self.hs, dtype=np.float32))
            buf[rk][:, :, read_heads[0]:read_heads[-1] + 1] = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        return buf

    def values(self, tensor_id, positions, heads):
        """Exact float64 values (of the bf16 inputs) at global positions / heads: what the oracle is fed."""
        return inputs.from_bf16_bits(inputs.to_bf16_bits(inputs.tensor_at(self.seed, tensor_id, self.bs, positions, heads, self.hs)))

    def forward(self):
        usp = self.usp
        self.o = torch.zeros_like(self.q)
        self.lse = torch.zeros((self.N, self.bs, self.hq, self.Lq), dtype=torch.float32, device="cuda")
        ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(self.p, 1), dtype=torch.uint8, device="cuda")
        usp.usp_attn_fwd(self.p, self.q, self.k, self.v, self.o, self.lse, self.rank, self.rank + 1, ws)
        torch.cuda.synchronize()

    def seq_rows(self, buf, local_rows, heads_slice):
        """Rows of the rank's ring block (local indices) gathered from a seq-layout buffer -> float64 [bs, rows, heads, hs]."""
        out = []
        for i in local_rows:
            shard = self.r * self.U + int(i) // self.n
            out.append(buf[shard, :, int(i) % self.n, heads_slice, :])
        return to_f64(torch.stack(out, dim=1))

    def sample_rows(self, rng, count, tile=256):
        """Uniform sample of local rows plus the first/last row of each zigzag chunk and of some tiles."""
        c = self.Lq // 2 if self.zigzag and self.R > 1 else self.Lq
        must = {0, self.Lq - 1, c - 1, c % self.Lq, tile - 1, tile, self.Lq - tile, self.Lq - tile - 1}
        rows = set(int(x) for x in rng.choice(self.Lq, size=min(count, self.Lq), replace=False)) | {m for m in must if 0 <= m < self.Lq}
        return np.array(sorted(rows), dtype=np.int64)
