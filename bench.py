#!/usr/bin/env python3
"""Benchmark of the one-rank USP attention forward on one MI355X.

A "step" is one pass of Algorithm 1's forward for ONE virtual rank of the workload:
all-to-all of Q, K, V (seq -> head layout), the ring loop of block attention with the LSE merge
and the all-to-all of O back -- all inputs resident in HBM before timing.

Default workload: the largest of the single-GPU configurations, the hybrid rank at long context
(the paper's LLaMA-3-8B, SP 16 example of Sec. 3): bs=1, L=212992, 32 Q heads / 8 KV heads, head size 128,
bf16, causal zigzag, Ulysses 8 x ring 2: rank 0 holds 4 Q heads + 1 KV head, 106496 queries against 2 K/V
blocks of 106496 keys.  The Ulysses-only rank (L=32768, Ulysses 8 x ring 1) is timed in the same run and reported
under "secondary" of the same JSON line.

Prints ONE JSON line: whole-step throughput in TFLOP/s (4*hs flop per visible (query, key) pair:
causal-effective under the mask), the dominant kernel's roofline (block attention vs the bf16 dense MFMA peak),
the HBM-bound kernels' GB/s, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak
PREWARM_MS = 80.0           # untimed load before the warm-up steps, see time_step()
DEFAULT_WORKLOAD = "hybrid_u8r2_L212992"
SECONDARY_WORKLOAD = "ulysses8_L32768"
# rocprofv3 counter figures per workload (HBM-side bytes and sustained clock of the attention launch), written by
# `python -m paper_2405_07719_amd.profile_summary` from the profiling runs described in profiles/*.md
MEASURED_JSON = os.path.join(ROOT, "profiles", "measured.json")

WORKLOADS = {
    # name: (bs, L, hc, hk, hs, U, R, timed rank, causal)
    "ulysses8_L32768": (1, 32768, 32, 8, 128, 8, 1, 0, True),
    "ring8_L32768": (1, 32768, 32, 8, 128, 1, 8, 0, True),
    "hybrid_u8r2_L212992": (1, 212992, 32, 8, 128, 8, 2, 0, True),
    "train_u2r4_L65536": (1, 65536, 32, 8, 128, 2, 4, 0, True),
    # the other head structures of the paper's benchmarks (parity cases with a throughput figure beside them)
    "mha_u8_L32768": (1, 32768, 32, 32, 128, 8, 1, 0, True),         # LLAMA2-7B-like: every Q head has its own KV head
    "mqa_ring8_L32768": (1, 32768, 32, 1, 128, 1, 8, 0, True),       # one KV head: Ulysses cannot split it, ring only
    "noncausal_u8_L32768": (1, 32768, 32, 8, 128, 8, 1, 0, False),   # bidirectional (DiT-style) attention
    "hs64_u8_L32768": (1, 32768, 32, 8, 64, 8, 1, 0, True),          # head size 64
}
# sampled query rows per head for the oracle leg: about 10-20 s of fp64 NumPy on 16 cores (every row meets all L keys)
CPU_ROWS = {"hybrid_u8r2_L212992": 2048, "train_u2r4_L65536": 8192}


def pairs_per_head(L, R, causal):
    """Visible (query, key) pairs of one ring rank's rows: every key without a mask, c^2 (2R-1) + c (c+1) under
    the causal mask with the zigzag split."""
    if not causal:
        return (L // R) * L
    c = L // (2 * R)
    return c * c * (2 * R - 1) + c * (c + 1)


def event_ms(fn, iters):
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def measured_for(workload):
    """The tracked counter figures of a workload (None when it has not been profiled)."""
    try:
        with open(MEASURED_JSON) as f:
            return json.load(f).get(workload)
    except (OSError, ValueError):
        return None


class Workload:
    """Seeded inputs of one workload, resident on the GPU, and the timed legs over them."""

    def __init__(self, name, rank=None, seed=1001):
        import numpy as np
        import torch

        import paper_2405_07719_amd as usp
        from paper_2405_07719_amd import inputs
        self.np, self.torch, self.usp, self.inputs = np, torch, usp, inputs
        self.name, self.seed = name, seed
        bs, L, hc, hk, hs, U, R, rk, causal = WORKLOADS[name]
        self.bs, self.L, self.hc, self.hk, self.hs, self.U, self.R, self.causal = bs, L, hc, hk, hs, U, R, causal
        self.N = U * R
        self.rank = rk if rank is None else rank
        self.p = usp.problem(bs, L, hc, hk, hs, U, R, causal, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
        self.r, self.u = divmod(self.rank, U)
        self.hq, self.hkv, self.Lq, self.n = hc // U, hk // U, L // R, L // self.N
        self.q_heads = np.arange(self.u * self.hq, (self.u + 1) * self.hq)
        self.kv_heads = np.arange(self.u * self.hkv, (self.u + 1) * self.hkv)
        # seeded inputs, materialised shard by shard from global coordinates (only the heads this rank reads)
        self.q = self.seq_buffer(inputs.TENSOR_Q, hc, self.q_heads)
        self.k = self.seq_buffer(inputs.TENSOR_K, hk, self.kv_heads)
        self.v = self.seq_buffer(inputs.TENSOR_V, hk, self.kv_heads)
        self.o = torch.zeros_like(self.q)
        self.lse = torch.zeros((self.N, bs, self.hq, self.Lq), dtype=torch.float32, device="cuda")
        self.ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(self.p, 1), dtype=torch.uint8, device="cuda")
        self.pairs = pairs_per_head(L, R, causal)
        self.flop = 4.0 * hs * self.pairs * self.hq * bs

    def shard_positions(self, rk):
        d, _ = self.usp.usp_local_positions(self.p, rk // self.U, rk % self.U)
        return self.np.array(d.positions(), dtype=self.np.int64)

    def seq_buffer(self, tensor_id, heads, read_heads):
        np, torch, inputs = self.np, self.torch, self.inputs
        buf = torch.zeros((self.N, self.bs, self.n, heads, self.hs), dtype=torch.bfloat16, device="cuda")
        for rk in range(self.N):
            bits = inputs.to_bf16_bits(inputs.tensor_at(self.seed, tensor_id, self.bs, self.shard_positions(rk), read_heads,
                                                        self.hs, dtype=np.float32))
            buf[rk][:, :, read_heads[0]:read_heads[-1] + 1] = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        return buf

    def config(self):
        return {"workload": self.name, "bs": self.bs, "L": self.L, "hc": self.hc, "hk": self.hk, "hs": self.hs,
                "ulysses": self.U, "ring": self.R, "causal": self.causal, "split": "zigzag", "timed_rank": self.rank,
                "flop_per_step": self.flop}

    def step(self):
        self.usp.usp_attn_fwd(self.p, self.q, self.k, self.v, self.o, self.lse, self.rank, self.rank + 1, self.ws)

    # ---- the whole step, wall clock around K steps
    def time_step(self, steps, warmup):
        """An idle MI355X needs a few tens of milliseconds of load before its clock settles (the first launches of
        the attention kernel run up to 20 % slow), so the chip is loaded with untimed steps for PREWARM_MS first; the
        W warm-up steps the caller asked for come after that."""
        torch = self.torch
        t_pre = time.perf_counter()
        while (time.perf_counter() - t_pre) * 1e3 < PREWARM_MS:
            self.step()
            torch.cuda.synchronize()
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        return ms, self.flop / (ms * 1e-3) / 1e12

    # ---- dominant kernel alone: the attention launch of one step, HIP events on the launch stream
    def roofline(self, steps, warmup, with_stepwise):
        usp, torch = self.usp, self.torch
        p, bs, hs, U, R, rank, r, u = self.p, self.bs, self.hs, self.U, self.R, self.rank, self.r, self.u
        hq, hkv, Lq, causal = self.hq, self.hkv, self.Lq, self.causal
        _, qd = usp.usp_local_positions(p, r, u)
        qh = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
        kh = torch.empty((R, bs, Lq, hkv, hs), dtype=torch.bfloat16, device="cuda")
        vh = torch.empty_like(kh)
        usp.usp_layout_a2a(p, self.hc, usp.USP_SEQ_TO_HEAD, self.q, qh.data_ptr() - rank * qh.numel() * 2, rank, rank + 1)
        for s in range(R):
            rk = s * U + u
            usp.usp_layout_a2a(p, self.hk, usp.USP_SEQ_TO_HEAD, self.k, kh[s].data_ptr() - rk * kh[s].numel() * 2, rk, rk + 1)
            usp.usp_layout_a2a(p, self.hk, usp.USP_SEQ_TO_HEAD, self.v, vh[s].data_ptr() - rk * vh[s].numel() * 2, rk, rk + 1)
        o_ring = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
        l_ring = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
        kds = [usp.usp_local_positions(p, (r - i) % R, u)[1] for i in range(R)]
        k_blocks = [kh[(r - i) % R] for i in range(R)]
        v_blocks = [vh[(r - i) % R] for i in range(R)]

        # what the step launches: the rank's whole ring loop over its R resident blocks in one launch, V staged in
        # key-tile-transposed layout by the all-to-all (a block [bs, Lq, hkv, hs] is the sequence layout of a
        # one-rank problem, so the same layout call transposes it here)
        pb = usp.problem(bs, Lq, hkv, hkv, hs, 1, 1, False, usp.USP_SPLIT_CONTIG, usp.USP_BF16)
        vt_blocks = []
        for vb_ in v_blocks:
            t = torch.empty((bs, hkv, (Lq + 63) // 64, hs, 64), dtype=torch.bfloat16, device="cuda")
            usp.usp_layout_a2a(pb, hkv, usp.USP_SEQ_TO_HEAD_VT, vb_, t, 0, 1)
            vt_blocks.append(t)

        # ... unless the step reads V where it lies: with Ulysses degree 1 a block in head layout is its shard, and
        # the library re-tiles V only when that pays (then its workspace holds the R re-tiled blocks)
        v_in_place = U == 1 and usp.usp_attn_fwd_workspace_bytes(p, 1) < sum(t.numel() * 2 for t in vt_blocks)

        def attn_only():
            if v_in_place:
                usp.usp_ring_attn_fwd(qh, k_blocks, v_blocks, kds, o_ring, l_ring, bs, Lq, Lq, hq, hkv, hs, 0.0, causal, qd,
                                      usp.USP_BF16, usp.USP_BF16)
            else:
                usp.usp_ring_attn_fwd_vt(qh, k_blocks, vt_blocks, kds, o_ring, l_ring, bs, Lq, Lq, hq, hkv, hs, 0.0, causal, qd)

        for _ in range(warmup):
            attn_only()
        attn_ms = event_ms(attn_only, steps)
        attn_tflops = self.flop / (attn_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "block_attn_fwd_mfma", "achieved": round(attn_tflops, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                "launches_per_step": 1, "avg_launch_ms": round(attn_ms, 4), "traffic": None,
                "algorithmic_bytes": float(2 * qh.numel() * 2 + 2 * kh.numel() * 2 + bs * hq * Lq * 4)}
        # HBM-side bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the same counter
        # reads for a plain 512 MiB copy) and the clock the box sustained under this kernel (GRBM_GUI_ACTIVE /
        # duration): from the tracked summary of the profiling runs of THIS workload, with the commit they were made at
        m = measured_for(self.name)
        if m is not None:
            roof["traffic"] = m.get("traffic_bytes")
            # the counters sit between the eight XCDs' private L2s and the fabric (Infinity Cache hits included): K
            # and V must enter every L2 that runs a workgroup of their KV head, so what a perfect schedule would
            # read here is Q once and K, V once per XCD, not once
            roof["traffic_floor_with_8_l2"] = float(roof["algorithmic_bytes"] + 7 * 2 * kh.numel() * 2)
            if m.get("clock_ghz"):
                roof["measured_clock_ghz"] = m["clock_ghz"]
                roof["frac_of_peak_at_measured_clock"] = round(attn_tflops / (256 * m["clock_ghz"] * 4096 / 1e3), 4)
            roof["counters_measured_at_commit"] = m.get("git_head")
        if with_stepwise and R > 1:
            # the same work as a ring that receives one block per step issues it
            o_parts = [torch.empty((bs, Lq, hq, hs), dtype=torch.float32, device="cuda") for _ in range(R)]
            l_parts = [torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda") for _ in range(R)]

            def attn_stepwise():
                for i in range(R):
                    usp.usp_block_attn_fwd(qh, k_blocks[i], v_blocks[i], o_parts[i], l_parts[i], bs, Lq, Lq, hq, hkv, hs,
                                           0.0, causal, qd, kds[i], usp.USP_BF16, usp.USP_FP32)
                usp.usp_lse_merge(o_parts, l_parts, o_ring, l_ring, bs, Lq, hq, hs, usp.USP_FP32, usp.USP_BF16)
            attn_stepwise()
            sms = event_ms(attn_stepwise, max(3, steps // 2))
            roof["stepwise_ring"] = {"launches": R + 1, "ms": round(sms, 4), "TFLOP/s": round(self.flop / (sms * 1e-3) / 1e12, 2),
                                     "note": "one usp_block_attn_fwd per block (fp32 partials) + usp_lse_merge"}
            del o_parts, l_parts
            if hasattr(usp, "usp_block_attn_fwd_state"):
                # the same ring with the running state (m, l, unnormalised O) carried from call to call: no partials
                state = torch.empty(usp.usp_block_attn_fwd_state_bytes(bs, Lq, hq, hs), dtype=torch.uint8, device="cuda")

                def attn_state():
                    for i in range(R):
                        usp.usp_block_attn_fwd_state(qh, k_blocks[i], v_blocks[i], state, o_ring, l_ring, bs, Lq, Lq, hq, hkv,
                                                     hs, 0.0, causal, qd, kds[i], i == 0, i == R - 1, usp.USP_BF16)
                attn_state()
                tms = event_ms(attn_state, max(3, steps // 2))
                roof["stepwise_ring_state"] = {"launches": R, "ms": round(tms, 4),
                                               "TFLOP/s": round(self.flop / (tms * 1e-3) / 1e12, 2),
                                               "note": "one usp_block_attn_fwd_state per block, running state in and out"}
        return roof

    # ---- HBM-bound legs: the all-ranks layout transform of this workload
    def layout_legs(self, steps):
        usp, torch = self.usp, self.torch
        extras = {}
        q_head_all = torch.empty((self.N, self.bs, self.Lq, self.hq, self.hs), dtype=torch.bfloat16, device="cuda")
        seq_back = torch.empty_like(self.q)

        def a2a_q():
            usp.usp_layout_a2a(self.p, self.hc, usp.USP_SEQ_TO_HEAD, self.q, q_head_all, 0, self.N)

        def a2a_o():
            usp.usp_layout_a2a(self.p, self.hc, usp.USP_HEAD_TO_SEQ, q_head_all, seq_back, 0, self.N)
        for name, fn in (("layout_a2a_seq_to_head", a2a_q), ("layout_a2a_head_to_seq", a2a_o)):
            fn()
            ms = event_ms(fn, max(steps, 20))
            nbytes = 2.0 * self.q.numel() * 2
            gbs = nbytes / (ms * 1e-3) / 1e9
            extras[name] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes": nbytes, "ms": round(ms, 4),
                            "shape": f"all {self.N} ranks, Q [{self.N},{self.bs},{self.n},{self.hc},{self.hs}] bf16"}
        return extras

    # ---- backward of the same rank (usp_attn_bwd): 2.5 x the forward flop by the usual accounting
    def backward(self, steps):
        usp, torch, inputs = self.usp, self.torch, self.inputs
        p, rank, flop = self.p, self.rank, self.flop
        d_o = self.seq_buffer(inputs.TENSOR_DO, self.hc, self.q_heads)
        dq, dk, dv = torch.zeros_like(self.q), torch.zeros_like(self.k), torch.zeros_like(self.v)
        n_plain, n_ds = usp.usp_attn_bwd_workspace_bytes(p, 1), usp.usp_attn_bwd_workspace_bytes_with_ds(p, 1)
        # the larger workspace lets the dK/dV kernel keep dS for the dQ kernel (5 products per tile pair instead of
        # 7): timed as well when it fits in 70 % of the free memory (equal sizes: dS is not kept at this head size)
        with_ds = n_plain < n_ds <= int(torch.cuda.mem_get_info()[0] * 0.7)
        ws_b = torch.empty(n_ds if with_ds else n_plain, dtype=torch.uint8, device="cuda")

        def bwd(nbytes=n_plain):
            usp.usp_attn_bwd(p, self.q, self.k, self.v, self.o, self.lse, d_o, dq, dk, dv, rank, rank + 1, ws_b, nbytes)
        bwd()
        bms = event_ms(bwd, max(3, steps // 4))
        out = {"ms_per_step": round(bms, 4), "value": round(2.5 * flop / (bms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
               "frac_of_mfma_peak": round(2.5 * flop / (bms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "workspace_bytes": n_plain,
               "note": "whole usp_attn_bwd of the timed rank (all-to-alls, delta, dQ and dK/dV kernels, conversion)"}
        if with_ds:
            bwd(n_ds)
            dms = event_ms(lambda: bwd(n_ds), max(3, steps // 4))
            out["with_stored_ds"] = {
                "ms_per_step": round(dms, 4), "value": round(2.5 * flop / (dms * 1e-3) / 1e12, 2),
                "frac_of_mfma_peak": round(2.5 * flop / (dms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "workspace_bytes": n_ds,
                "note": "same call with the larger workspace: dS written by the dK/dV kernel and read by the dQ kernel"}
        return out

    # ---- CPU oracle on a bounded sample of the same workload (rows of the timed rank), with parity
    def cpu_baseline_and_parity(self, n_rows):
        np, torch, inputs = self.np, self.torch, self.inputs
        from oracle import usp_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([t.get("num_threads", 1) for t in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        L, U, R, n, hq, bs, hs, Lq = self.L, self.U, self.R, self.n, self.hq, self.bs, self.hs, self.Lq
        # rows are picked, and the step's inputs were placed, by Algorithm 2: the ORACLE's map here, which must be
        # the map the inputs were placed with (the library's) for every shard the step read
        for rk in range(self.N):
            assert np.array_equal(self.shard_positions(rk), orc.zigzag_positions(L, R, U, rk // U, rk % U, True)), \
                f"the library's Algorithm-2 positions of rank {rk} differ from the oracle's"
        blk = orc.ring_block_positions(L, R, self.r, True)
        rng = np.random.default_rng(self.seed)
        rows_local = np.sort(rng.choice(Lq, size=min(n_rows, Lq), replace=False))
        rows_pos = blk[rows_local]
        allpos = np.arange(L)
        gen = lambda tid, pos, heads: inputs.from_bf16_bits(inputs.to_bf16_bits(inputs.tensor_at(self.seed, tid, bs, pos, heads, hs)))
        qs = gen(inputs.TENSOR_Q, rows_pos, self.q_heads)
        kg = gen(inputs.TENSOR_K, allpos, self.kv_heads)
        vg = gen(inputs.TENSOR_V, allpos, self.kv_heads)
        t0 = time.perf_counter()
        ref_o, ref_l = orc.attention_rows(qs, rows_pos, kg, vg, self.causal)
        cpu_s = time.perf_counter() - t0
        sample_pairs = (float((rows_pos + 1).sum()) if self.causal else float(rows_pos.size) * L) * hq * bs
        base = {"value": round(4.0 * hs * sample_pairs / cpu_s / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores),
                "kind": "oracle", "seconds": round(cpu_s, 2), "pairs_per_s": round(sample_pairs / cpu_s, 1),
                "extrapolated_full_step_seconds": round(cpu_s * (self.pairs * hq * bs) / sample_pairs, 1),
                "sample": f"{rows_local.size} uniformly sampled query rows x {hq} heads of the timed rank, all {L} keys, "
                          f"fp64 NumPy; same flop accounting (4*hs per visible pair)"}
        # parity of the timed step's output on the sampled rows.  Local row i of the ring block lives in shard
        # u' = i // n of ring row r, at offset i % n (Algorithm 1's all-to-all gathers ascending Ulysses ranks)
        rows_t = torch.from_numpy(rows_local).cuda()
        got_bits = self.o[self.r * U + rows_t // n, :, rows_t % n][:, :, self.u * hq:(self.u + 1) * hq]   # [rows, bs, hq, hs]
        got_rows = inputs.from_bf16_bits(got_bits.cpu().view(torch.int16).numpy().view(np.uint16)).reshape(got_bits.shape)
        got_rows = np.transpose(got_rows, (1, 0, 2, 3))
        lse_rows = self.lse[self.rank].cpu().double().numpy()[:, :, rows_local]
        parity = {"max_abs_o": float(np.max(np.abs(got_rows - ref_o))), "max_abs_lse": float(np.max(np.abs(lse_rows - ref_l))),
                  "rows": int(rows_local.size), "tolerance": {"o": 2e-2, "lse": 1e-3},
                  "positions": "oracle's Algorithm 2 map (checked equal to the library's for every shard)"}
        return base, parity


def merge_leg(usp, torch, steps, hs=128):
    """An 8-way merge at the ring-only rank's shape (working set far beyond the 256 MiB on-die cache)."""
    mp, mL, mh = 8, 4096, 32
    parts = [torch.randn((1, mL, mh, hs), dtype=torch.float32, device="cuda") for _ in range(mp)]
    lparts = [torch.randn((1, mh, mL), dtype=torch.float32, device="cuda") for _ in range(mp)]
    mo = torch.empty((1, mL, mh, hs), dtype=torch.bfloat16, device="cuda")
    ml = torch.empty((1, mh, mL), dtype=torch.float32, device="cuda")

    def merge():
        usp.usp_lse_merge(parts, lparts, mo, ml, 1, mL, mh, hs, usp.USP_FP32, usp.USP_BF16)
    merge()
    ms = event_ms(merge, max(steps, 20))
    nbytes = mp * (mL * mh * hs * 4.0 + mL * mh * 4.0) + mL * mh * hs * 2.0 + mL * mh * 4.0
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
            "bytes": nbytes, "ms": round(ms, 4), "shape": f"{mp} fp32 partials [1,{mL},{mh},{hs}] -> bf16 (ring-only rank)"}


def calibration_leg(torch):
    """What the matrix core delivers on this machine: a pure MFMA loop, and a loop with the forward kernel's steady-state
    instruction mix (MFMA + exp2 + LDS operand reads, random operand bits, no global memory)."""
    from paper_2405_07719_amd import calib as usp_calib
    sink = torch.empty(usp_calib.USP_CALIB_SINK_BYTES, dtype=torch.uint8, device="cuda")
    calib = {}
    for mode, name in ((0, "pure_mfma"), (1, "attention_mix_random_operands")):
        cflop = usp_calib.usp_calib_mfma(mode, 2000, sink)
        cms = event_ms(lambda: usp_calib.usp_calib_mfma(mode, 2000, sink), 5)
        calib[name] = {"TFLOP/s": round(cflop / (cms * 1e-3) / 1e12, 1), "ms": round(cms, 3)}
    calib["note"] = ("context for roofline.frac: loops without global-memory traffic, masks or bookkeeping; "
                     "256 workgroups x 8 waves, v_mfma_f32_32x32x16_bf16")
    return calib


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--rank", type=int, default=None,
                    help="virtual rank to time (default: ring rank 0, Ulysses rank 0; ring rank R-1 has the same pair "
                         "count but a different tile geometry)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-extras", action="store_true", help="skip the layout / merge bandwidth and calibration legs")
    ap.add_argument("--cpu-rows", type=int, default=None, help="sampled query rows per head for the oracle leg")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward (usp_attn_bwd) timing leg")
    ap.add_argument("--no-secondary", action="store_true",
                    help=f"skip the secondary block ({SECONDARY_WORKLOAD}, timed when the default workload is run)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 512 MiB device copies: the known-size kernel that scales FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (ring and Ulysses ranks are simulated locally); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2405_07719_amd as usp

    usp.load()   # no fallback: raises if the HIP library is missing
    torch.cuda.set_device(0)
    N = WORKLOADS[args.workload][5] * WORKLOADS[args.workload][6]
    if args.rank is not None and not 0 <= args.rank < N:
        print(f"bench.py: --rank must be in [0, {N})", file=sys.stderr)
        sys.exit(2)

    w = Workload(args.workload, args.rank)
    ms_per_step, value = w.time_step(args.steps, args.warmup)
    out = {
        "metric": "one-rank USP attention TFLOP/s (bf16 causal fwd) + % MFMA peak; a2a GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "prewarm_ms": PREWARM_MS, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": w.config(),
        "roofline": w.roofline(args.steps, args.warmup, not args.no_extras),
    }
    if not args.no_extras:
        out["hbm_kernels"] = w.layout_legs(args.steps)
        out["hbm_kernels"]["lse_merge"] = merge_leg(usp, torch, args.steps)
        out["mfma_calibration"] = calibration_leg(torch)
    if not args.no_backward:
        out["backward"] = w.backward(args.steps)
    if args.copy_calibration:
        src = torch.empty(512 * 2**20, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        rows = args.cpu_rows or CPU_ROWS.get(args.workload, 16384)
        out["cpu_baseline"], out["parity"] = w.cpu_baseline_and_parity(rows)
    del w
    torch.cuda.empty_cache()

    # ---- the Ulysses-only rank (configs[1]) in the same run: whole step, its attention launch, layout legs, backward
    if args.workload == DEFAULT_WORKLOAD and not args.no_secondary:
        s = Workload(SECONDARY_WORKLOAD)
        sms, sval = s.time_step(args.steps, args.warmup)
        sec = {"value": round(sval, 2), "unit": "TFLOP/s", "ms_per_step": round(sms, 4), "steps": args.steps,
               "warmup": args.warmup, "config": s.config(), "roofline": s.roofline(args.steps, args.warmup, False)}
        if not args.no_extras:
            sec["hbm_kernels"] = s.layout_legs(args.steps)
        if not args.no_backward:
            sec["backward"] = s.backward(args.steps)
        if not args.no_cpu_baseline:
            _, sec["parity"] = s.cpu_baseline_and_parity(1024)
        out["secondary"] = {SECONDARY_WORKLOAD: sec}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
