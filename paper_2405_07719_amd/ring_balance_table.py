"""Per-rank compute time of USP attention for the grid of the paper's attention benchmark (Sec. 5, the two
forward-only tables: sequence length x Ulysses degree, basic ring vs load-balanced ring), on ONE GPU.

For every (L, U) with U * R = 8 and both ways of cutting ring blocks from the sequence (contiguous = "basic-ring",
zigzag = "lb-ring"), each ring rank's forward (`usp_attn_fwd` of virtual rank (r, 0): all-to-alls, ring loop,
merge) is timed alone; a synchronous 8-GPU step would take the maximum over the ring ranks, so the table prints
1 / max as "compute-only iterations per second" beside the max/min ratio that shows the imbalance of the even
split.  No communication is modelled.  Inputs are seeded N(0,1) tensors made on the device (values do not change
the timing); this is a measurement script, not a parity test.

    python -m paper_2405_07719_amd.ring_balance_table [--seqlens 8192 16384 32768 131072] [--iters 5] [--backward]

--backward adds, for the load-balanced split, the time of `usp_attn_bwd` of ring rank 0 (all ring ranks do the same
work there) and its rate by the usual 2.5 x forward flop accounting.
"""
from __future__ import annotations

import argparse

import torch

import paper_2405_07719_amd as usp


def time_rank(p, q, k, v, o, lse, ws, rank, iters):
    usp.usp_attn_fwd(p, q, k, v, o, lse, rank, rank + 1, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        usp.usp_attn_fwd(p, q, k, v, o, lse, rank, rank + 1, ws)
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seqlens", type=int, nargs="+", default=[8192, 16384, 32768, 131072])
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--backward", action="store_true", help="also time usp_attn_bwd of ring rank 0, lb split")
    args = ap.parse_args()
    usp.load()
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda").manual_seed(1234)
    bs, hc, hk, hs, N = 1, 32, 8, 128, 8
    print("| seqlen | ulysses | ring | basic: max ms | basic: max/min | basic it/s | lb: max ms | lb: max/min | lb it/s |"
          + (" lb: bwd ms | lb: bwd TFLOP/s |" if args.backward else ""))
    print("|---|---|---|---|---|---|---|---|---|" + ("---|---|" if args.backward else ""))
    for L in args.seqlens:
        q = torch.randn((N, bs, L // N, hc, hs), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        k = torch.randn((N, bs, L // N, hk, hs), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        v = torch.randn((N, bs, L // N, hk, hs), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        o = torch.empty_like(q)
        for U in (8, 4, 2, 1):
            R = N // U
            cells = []
            for split in (usp.USP_SPLIT_CONTIG, usp.USP_SPLIT_ZIGZAG):
                p = usp.problem(bs, L, hc, hk, hs, U, R, True, split, usp.USP_BF16)
                lse = torch.empty((N, bs, hc // U, L // R), dtype=torch.float32, device="cuda")
                ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, 1), dtype=torch.uint8, device="cuda")
                ms = [time_rank(p, q, k, v, o, lse, ws, r * U, args.iters) for r in range(R)]
                cells += [f"{max(ms):.3f}", f"{max(ms) / min(ms):.2f}", f"{1e3 / max(ms):.1f}"]
                if args.backward and split == usp.USP_SPLIT_ZIGZAG:
                    usp.usp_attn_fwd(p, q, k, v, o, lse, 0, 1, ws)      # O and LSE of rank 0 for its backward
                    d_o, dq, dk, dv = torch.randn_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
                    wb = torch.empty(usp.usp_attn_bwd_workspace_bytes(p, 1), dtype=torch.uint8, device="cuda")
                    bwd = lambda: usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, 0, 1, wb)
                    bwd()
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(args.iters):
                        bwd()
                    e1.record()
                    e1.synchronize()
                    bms = e0.elapsed_time(e1) / args.iters
                    c = L // (2 * R)
                    flop = 2.5 * 4 * hs * (c * c * (2 * R - 1) + c * (c + 1)) * (hc // U) * bs
                    cells += [f"{bms:.3f}", f"{flop / bms / 1e9:.0f}"]
                    del d_o, dq, dk, dv, wb
            print(f"| {L} | {U} | {R} | " + " | ".join(cells) + " |", flush=True)
        del q, k, v, o


if __name__ == "__main__":
    main()
