#!/usr/bin/env python3
"""Benchmark of the one-rank USP attention forward on one MI355X.

A "step" is one pass of Algorithm 1's forward for ONE virtual rank of the workload:
all-to-all of Q, K, V (seq -> head layout), the ring loop of block attention, the LSE merge
(when ring > 1) and the all-to-all of O back -- all inputs resident in HBM before timing.

Default workload (the configuration the headline metric is quoted on): the Ulysses-only rank
of a LLaMA-3-8B-shaped attention, bs=1, L=32768, 32 Q heads / 8 KV heads, head size 128, bf16,
causal, Ulysses 8 x ring 1: rank 0 holds 4 Q heads + 1 KV head over the full sequence.

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

# rocprofv3 --pmc FETCH_SIZE (x2, the factor a plain copy of known size gives) + WRITE_SIZE, KiB -> bytes, per
# launch of the block-attention kernel
# (copy calibration: a 524288 KiB copy reads FETCH_SIZE 262158, WRITE_SIZE 524288)
PREWARM_MS = 80.0          # untimed load before the warm-up steps, see main()
MEASURED_CLOCK_GHZ = 2.06   # block_attn_fwd_mfma on the default workload, see profiles/clock_cycles_ulysses8_L32768.md
MEASURED_TRAFFIC_BYTES = {"ulysses8_L32768": round((150998 * (524288 / 262156) + 40985 * (524288 / 524288)) * 1024.0)}

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="ulysses8_L32768", choices=sorted(WORKLOADS))
    ap.add_argument("--rank", type=int, default=None,
                    help="virtual rank to time (default: ring rank 0, Ulysses rank 0; ring rank R-1 has the same pair "
                         "count but a different tile geometry)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-extras", action="store_true", help="skip the layout / merge bandwidth legs")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="sampled query rows per head for the oracle leg")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward (usp_attn_bwd) timing leg")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 512 MiB device copies: the known-size kernel that scales FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (ring and Ulysses ranks are simulated locally); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2405_07719_amd as usp
    from paper_2405_07719_amd import inputs

    usp.load()   # no fallback: raises if the HIP library is missing
    torch.cuda.set_device(0)
    bs, L, hc, hk, hs, U, R, rank, causal = WORKLOADS[args.workload]
    N = U * R
    if args.rank is not None:
        if not 0 <= args.rank < N:
            print(f"bench.py: --rank must be in [0, {N})", file=sys.stderr)
            sys.exit(2)
        rank = args.rank
    seed = 1001
    p = usp.problem(bs, L, hc, hk, hs, U, R, causal, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    r, u = divmod(rank, U)
    hq, hkv, Lq, n = hc // U, hk // U, L // R, L // N

    # ---- seeded inputs, materialised shard by shard from global coordinates (heads this rank reads)
    def shard_positions(rk):
        d, _ = usp.usp_local_positions(p, rk // U, rk % U)
        return np.array(d.positions(), dtype=np.int64)

    def seq_buffer(tensor_id, heads, read_heads):
        buf = torch.zeros((N, bs, n, heads, hs), dtype=torch.bfloat16, device="cuda")
        for rk in range(N):
            bits = inputs.to_bf16_bits(inputs.tensor_at(seed, tensor_id, bs, shard_positions(rk), read_heads, hs, dtype=np.float32))
            buf[rk][:, :, read_heads[0]:read_heads[-1] + 1] = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        return buf

    q_heads = np.arange(u * hq, (u + 1) * hq)
    kv_heads = np.arange(u * hkv, (u + 1) * hkv)
    q = seq_buffer(inputs.TENSOR_Q, hc, q_heads)
    k = seq_buffer(inputs.TENSOR_K, hk, kv_heads)
    v = seq_buffer(inputs.TENSOR_V, hk, kv_heads)
    o = torch.zeros_like(q)
    lse = torch.zeros((N, bs, hq, Lq), dtype=torch.float32, device="cuda")
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, 1), dtype=torch.uint8, device="cuda")

    def step():
        usp.usp_attn_fwd(p, q, k, v, o, lse, rank, rank + 1, ws)

    # An idle MI355X needs a few tens of milliseconds of load before its clock settles (the first launches of the
    # attention kernel run up to 20 % slow), so the chip is loaded with untimed steps for PREWARM_MS first; the W
    # warm-up steps the caller asked for come after that.
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < PREWARM_MS:
        step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    pairs = pairs_per_head(L, R, causal)
    flop = 4.0 * hs * pairs * hq * bs
    value = flop / (ms_per_step * 1e-3) / 1e12

    # ---- dominant kernel alone: the block-attention launches of one step, HIP events on the launch stream
    _, qd = usp.usp_local_positions(p, r, u)
    qh = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
    kh = torch.empty((R, bs, Lq, hkv, hs), dtype=torch.bfloat16, device="cuda")
    vh = torch.empty_like(kh)
    usp.usp_layout_a2a(p, hc, usp.USP_SEQ_TO_HEAD, q, qh.data_ptr() - rank * qh.numel() * 2, rank, rank + 1)
    for s in range(R):
        rk = s * U + u
        usp.usp_layout_a2a(p, hk, usp.USP_SEQ_TO_HEAD, k, kh[s].data_ptr() - rk * kh[s].numel() * 2, rk, rk + 1)
        usp.usp_layout_a2a(p, hk, usp.USP_SEQ_TO_HEAD, v, vh[s].data_ptr() - rk * vh[s].numel() * 2, rk, rk + 1)
    o_ring = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
    l_ring = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    kds = [usp.usp_local_positions(p, (r - i) % R, u)[1] for i in range(R)]
    k_blocks = [kh[(r - i) % R] for i in range(R)]
    v_blocks = [vh[(r - i) % R] for i in range(R)]

    def attn_only():      # what the step launches: the rank's whole ring loop, R resident blocks, one launch
        usp.usp_ring_attn_fwd(qh, k_blocks, v_blocks, kds, o_ring, l_ring, bs, Lq, Lq, hq, hkv, hs, 0.0, causal, qd,
                              usp.USP_BF16, usp.USP_BF16)

    for _ in range(args.warmup):
        attn_only()
    attn_ms = event_ms(attn_only, args.steps)
    attn_tflops = flop / (attn_ms * 1e-3) / 1e12
    stepwise = None
    if R > 1 and not args.no_extras:
        # the same work as a real ring would issue it: one launch per arriving block with fp32 partials, then the merge
        o_parts = [torch.empty((bs, Lq, hq, hs), dtype=torch.float32, device="cuda") for _ in range(R)]
        l_parts = [torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda") for _ in range(R)]

        def attn_stepwise():
            for i in range(R):
                usp.usp_block_attn_fwd(qh, k_blocks[i], v_blocks[i], o_parts[i], l_parts[i], bs, Lq, Lq, hq, hkv, hs,
                                       0.0, causal, qd, kds[i], usp.USP_BF16, usp.USP_FP32)
            usp.usp_lse_merge(o_parts, l_parts, o_ring, l_ring, bs, Lq, hq, hs, usp.USP_FP32, usp.USP_BF16)
        attn_stepwise()
        sms = event_ms(attn_stepwise, max(3, args.steps // 2))
        stepwise = {"launches": R + 1, "ms": round(sms, 4), "TFLOP/s": round(flop / (sms * 1e-3) / 1e12, 2),
                    "note": "one usp_block_attn_fwd per block (fp32 partials) + usp_lse_merge"}
        del o_parts, l_parts
    # HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this workload, each scaled by what
    # the same counter reads for a plain 512 MiB copy (FETCH_SIZE reads half the bytes, WRITE_SIZE all of them):
    # see profiles/traffic_pmc_ulysses8_L32768.md.  Only known for the default workload.
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload)
    roofline = {"bound": "mfma", "kernel": "block_attn_fwd_mfma", "achieved": round(attn_tflops, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                "launches_per_step": 1, "avg_launch_ms": round(attn_ms, 4), "traffic": traffic,
                "algorithmic_bytes": float(2 * qh.numel() * 2 + 2 * kh.numel() * 2 + bs * hq * Lq * 4)}
    if traffic is not None:
        # the counters sit between the eight XCDs' private L2s and the fabric (Infinity Cache hits included): K and V
        # must enter every L2 that runs a workgroup of their KV head, so what a perfect schedule would read here is
        # Q once and K, V once per XCD, not once
        kv_bytes = 2 * kh.numel() * 2
        roofline["traffic_floor_with_8_l2"] = float(roofline["algorithmic_bytes"] + 7 * kv_bytes)
        roofline["traffic_note"] = ("fills of the eight private L2s (the 16 MiB of K and V stay in the 256 MiB Infinity "
                                    "Cache: cache-to-cache traffic, 0.36 TB/s, not a bound)")
    if stepwise is not None:
        roofline["stepwise_ring"] = stepwise
    # the same fraction against CUs x the clock the box sustained under this kernel (GRBM_GUI_ACTIVE / duration in
    # profiles/clock_cycles_ulysses8_L32768.md) x 4096 bf16 MFMA flop per CU and cycle
    roofline["frac_of_peak_at_measured_clock"] = round(attn_tflops / (256 * MEASURED_CLOCK_GHZ * 4096 / 1e3), 4)
    roofline["measured_clock_ghz"] = MEASURED_CLOCK_GHZ

    out = {
        "metric": "one-rank USP attention TFLOP/s (bf16 causal fwd) + % MFMA peak; a2a GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "prewarm_ms": PREWARM_MS, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "bs": bs, "L": L, "hc": hc, "hk": hk, "hs": hs, "ulysses": U, "ring": R,
                   "causal": causal, "split": "zigzag", "timed_rank": rank, "flop_per_step": flop},
        "roofline": roofline,
    }

    # ---- HBM-bound legs: the all-ranks layout transform of this workload, and an 8-way merge at the
    #      ring-only rank's shape (working sets far beyond the 256 MiB on-die cache)
    if not args.no_extras:
        extras = {}
        q_head_all = torch.empty((N, bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
        seq_back = torch.empty_like(q)

        def a2a_q():
            usp.usp_layout_a2a(p, hc, usp.USP_SEQ_TO_HEAD, q, q_head_all, 0, N)

        def a2a_o():
            usp.usp_layout_a2a(p, hc, usp.USP_HEAD_TO_SEQ, q_head_all, seq_back, 0, N)
        for name, fn in (("layout_a2a_seq_to_head", a2a_q), ("layout_a2a_head_to_seq", a2a_o)):
            fn()
            ms = event_ms(fn, max(args.steps, 20))
            nbytes = 2.0 * q.numel() * 2
            gbs = nbytes / (ms * 1e-3) / 1e9
            extras[name] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes": nbytes, "ms": round(ms, 4),
                            "shape": f"all {N} ranks, Q [{N},{bs},{n},{hc},{hs}] bf16"}
        del q_head_all, seq_back
        mp, mL, mh = 8, 4096, 32
        parts = [torch.randn((1, mL, mh, hs), dtype=torch.float32, device="cuda") for _ in range(mp)]
        lparts = [torch.randn((1, mh, mL), dtype=torch.float32, device="cuda") for _ in range(mp)]
        mo = torch.empty((1, mL, mh, hs), dtype=torch.bfloat16, device="cuda")
        ml = torch.empty((1, mh, mL), dtype=torch.float32, device="cuda")

        def merge():
            usp.usp_lse_merge(parts, lparts, mo, ml, 1, mL, mh, hs, usp.USP_FP32, usp.USP_BF16)
        merge()
        ms = event_ms(merge, max(args.steps, 20))
        nbytes = mp * (mL * mh * hs * 4.0 + mL * mh * 4.0) + mL * mh * hs * 2.0 + mL * mh * 4.0
        gbs = nbytes / (ms * 1e-3) / 1e9
        extras["lse_merge"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                               "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes": nbytes, "ms": round(ms, 4),
                               "shape": f"{mp} fp32 partials [1,{mL},{mh},{hs}] -> bf16 (ring-only rank)"}
        del parts, lparts
        out["hbm_kernels"] = extras

        # ---- what the matrix core delivers on this machine: a pure MFMA loop, and a loop with the forward kernel's
        #      steady-state instruction mix (MFMA + exp2 + LDS operand reads, random operand bits, no global memory)
        sink = torch.empty(usp.USP_CALIB_SINK_BYTES, dtype=torch.uint8, device="cuda")
        calib = {}
        for mode, name in ((0, "pure_mfma"), (1, "attention_mix_random_operands")):
            cflop = usp.usp_calib_mfma(mode, 2000, sink)
            cms = event_ms(lambda: usp.usp_calib_mfma(mode, 2000, sink), 5)
            calib[name] = {"TFLOP/s": round(cflop / (cms * 1e-3) / 1e12, 1), "ms": round(cms, 3)}
        calib["note"] = ("context for roofline.frac: loops without global-memory traffic, masks or bookkeeping; "
                         "256 workgroups x 8 waves, v_mfma_f32_32x32x16_bf16")
        out["mfma_calibration"] = calib
        del sink

    # ---- backward of the same rank (usp_attn_bwd): 2.5 x the forward flop by the usual accounting
    if not args.no_backward:
        d_o = seq_buffer(inputs.TENSOR_DO, hc, q_heads)
        dq, dk, dv = torch.zeros_like(q), torch.zeros_like(k), torch.zeros_like(v)
        n_plain, n_ds = usp.usp_attn_bwd_workspace_bytes(p, 1), usp.usp_attn_bwd_workspace_bytes_with_ds(p, 1)
        # the larger workspace lets the dK/dV kernel keep dS for the dQ kernel (5 products per tile pair instead of
        # 7): timed as well when it fits in a quarter of the free memory
        with_ds = n_plain < n_ds <= torch.cuda.mem_get_info()[0] // 4   # equal sizes: dS is not kept at this head size
        ws_b = torch.empty(n_ds if with_ds else n_plain, dtype=torch.uint8, device="cuda")

        def bwd(nbytes=n_plain):
            usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, rank, rank + 1, ws_b, nbytes)
        bwd()
        bms = event_ms(bwd, max(3, args.steps // 4))
        out["backward"] = {"ms_per_step": round(bms, 4), "value": round(2.5 * flop / (bms * 1e-3) / 1e12, 2),
                           "unit": "TFLOP/s", "frac_of_mfma_peak": round(2.5 * flop / (bms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                           "workspace_bytes": n_plain,
                           "note": "whole usp_attn_bwd of the timed rank (all-to-alls, delta, dQ and dK/dV kernels, conversion)"}
        if with_ds:
            bwd(n_ds)
            dms = event_ms(lambda: bwd(n_ds), max(3, args.steps // 4))
            out["backward"]["with_stored_ds"] = {
                "ms_per_step": round(dms, 4), "value": round(2.5 * flop / (dms * 1e-3) / 1e12, 2),
                "frac_of_mfma_peak": round(2.5 * flop / (dms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                "workspace_bytes": n_ds,
                "note": "same call with the larger workspace: dS written by the dK/dV kernel and read by the dQ kernel"}
        del d_o, dq, dk, dv, ws_b

    if args.copy_calibration:
        src = torch.empty(512 * 2**20, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU oracle on a bounded sample of the same workload (rows of the timed rank), with parity
    if not args.no_cpu_baseline:
        from oracle import usp_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([t.get("num_threads", 1) for t in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        rng = np.random.default_rng(seed)
        blk = np.array(qd.positions(), dtype=np.int64)
        rows_local = np.sort(rng.choice(Lq, size=min(args.cpu_rows, Lq), replace=False))
        rows_pos = blk[rows_local]
        allpos = np.arange(L)
        qs = inputs.from_bf16_bits(inputs.to_bf16_bits(inputs.tensor_at(seed, inputs.TENSOR_Q, bs, rows_pos, q_heads, hs)))
        kg = inputs.from_bf16_bits(inputs.to_bf16_bits(inputs.tensor_at(seed, inputs.TENSOR_K, bs, allpos, kv_heads, hs)))
        vg = inputs.from_bf16_bits(inputs.to_bf16_bits(inputs.tensor_at(seed, inputs.TENSOR_V, bs, allpos, kv_heads, hs)))
        t0 = time.perf_counter()
        ref_o, ref_l = orc.attention_rows(qs, rows_pos, kg, vg, causal)
        cpu_s = time.perf_counter() - t0
        sample_pairs = (float((rows_pos + 1).sum()) if causal else float(rows_pos.size) * L) * hq * bs
        out["cpu_baseline"] = {"value": round(4.0 * hs * sample_pairs / cpu_s / 1e12, 5), "unit": "TFLOP/s",
                               "cores": int(cores), "kind": "oracle", "seconds": round(cpu_s, 2),
                               "pairs_per_s": round(sample_pairs / cpu_s, 1),
                               "extrapolated_full_step_seconds": round(cpu_s * (pairs * hq * bs) / sample_pairs, 1),
                               "sample": f"{rows_local.size} uniformly sampled query rows x {hq} heads of the timed rank, "
                                         f"all {L} keys, fp64 NumPy; same flop accounting (4*hs per visible pair)"}
        # parity of the timed step's output on the sampled rows (O comes back in seq layout: pick rank/rows)
        o_host = o.cpu().view(torch.int16).numpy().view(np.uint16)            # [N][bs][n][hc][hs]
        got = inputs.from_bf16_bits(o_host).reshape(N, bs, n, hc, hs)
        # local row i of the ring block lives in shard u' = i // n of ring row r, at offset i % n
        got_rows = np.stack([got[r * U + (i // n), :, i % n, u * hq:(u + 1) * hq, :] for i in rows_local], axis=1)
        lse_rows = lse[rank].cpu().double().numpy()[:, :, rows_local]
        out["parity"] = {"max_abs_o": float(np.max(np.abs(got_rows - ref_o))),
                         "max_abs_lse": float(np.max(np.abs(lse_rows - ref_l))), "rows": int(rows_local.size)}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
