"""GPU parity: backward of the block attention and of Algorithm 1, through the C ABI.

Tolerance (max-abs, from the benchmark spec): 5e-2 on dQ, dK, dV for the bf16 path.
"""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2405_07719_amd import inputs
from tests import usp_testlib as tl

pytestmark = pytest.mark.gpu
GRAD_TOL = 5e-2


def _desc(usp, t):
    return usp.usp_posdesc(*(list(t) + [0] * (4 - len(t))))


BWD_CASES = [
    # name, bs, Lq, Lk, hq, hkv, hs, causal, q desc, k desc, key-block cuts (local key ranges processed as separate steps)
    ("noncausal", 1, 320, 256, 4, 2, 128, False, None, None, [0, 256]),
    ("causal_diag_two_blocks", 1, 512, 512, 4, 2, 128, True, (0, 512), (0, 512), [0, 192, 512]),
    ("causal_ragged_gqa4", 2, 333, 333, 4, 1, 128, True, (0, 333), (0, 333), [0, 333]),
    ("zigzag_q_r1_all_keys", 1, 512, 2048, 4, 2, 128, True, (256, 256, 1536, 256), (0, 2048), [0, 700, 2048]),
    ("hs64", 1, 300, 300, 2, 2, 64, True, (0, 300), (0, 300), [0, 300]),
    # enough (key tile, KV head, batch) units that one workgroup walks both query heads of a group and stores its
    # dK/dV without atomics: first block overwrites, second block adds
    ("many_kv_units_plain_stores", 4, 96, 8192, 16, 8, 128, True, (8100, 96), (0, 8192), [0, 4096, 8192]),
    # multi-query group of 32 heads over 64 (key tile, batch) units: the heads are split 16 ways, two per workgroup,
    # and the workgroups of a key tile meet through atomic adds
    ("mqa_partial_head_split", 2, 64, 8192, 32, 1, 128, True, (8100, 64), (0, 8192), [0, 8192]),
]


@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_block_attn_bwd_sums_to_full_gradient(usp, case):
    _, bs, Lq, Lk, hq, hkv, hs, causal, qd, kd, cuts = case
    qdesc = _desc(usp, qd) if qd else None
    kdesc = _desc(usp, kd) if kd else None
    qpos = np.array(qdesc.positions()) if causal else np.arange(Lq)
    kpos = np.array(kdesc.positions()) if causal else np.arange(Lk)
    qs, qv = tl.gen(21, inputs.TENSOR_Q, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
    ks, kv = tl.gen(21, inputs.TENSOR_K, bs, np.arange(Lk), np.arange(hkv), hs, tl.BF16)
    vs, vv = tl.gen(21, inputs.TENSOR_V, bs, np.arange(Lk), np.arange(hkv), hs, tl.BF16)
    gs, gv = tl.gen(21, inputs.TENSOR_DO, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
    ref_dq, ref_dk, ref_dv = orc.attention_backward(qv, kv, vv, gv, causal, None, qpos, kpos)
    q, k, v, d_o = (tl.to_device(x, tl.BF16) for x in (qs, ks, vs, gs))
    o = torch.empty_like(q)
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_block_attn_fwd(q, k, v, o, lse, bs, Lq, Lk, hq, hkv, hs, 0.0, causal, qdesc, kdesc, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, Lq, hq, hs)
    # delta against its definition on the same (GPU) O
    torch.cuda.synchronize()
    d_ref = np.einsum("bihe,bihe->bhi", tl.to_f64(o), gv)
    assert tl.max_abs(tl.to_f64(delta), d_ref) <= 1e-3
    dq = torch.full((bs, Lq, hq, hs), float("nan"), dtype=torch.float32, device="cuda")
    dk = torch.full((bs, Lk, hkv, hs), float("nan"), dtype=torch.float32, device="cuda")
    dv = torch.full((bs, Lk, hkv, hs), float("nan"), dtype=torch.float32, device="cuda")
    for step, (a, b) in enumerate(zip(cuts, cuts[1:])):
        # key block [a, b): its own tensors, descriptor cut from the key descriptor, gradients into the block's rows
        if causal:
            kp = kpos[a:b]
            brk = np.nonzero(np.diff(kp) != 1)[0]
            if brk.size:
                n0 = int(brk[0]) + 1
                kdb = usp.usp_posdesc(int(kp[0]), n0, int(kp[n0]), b - a - n0)
            else:
                kdb = usp.usp_posdesc(int(kp[0]), b - a, 0, 0)
        else:
            kdb = None
        kb, vb = k[:, a:b].contiguous(), v[:, a:b].contiguous()
        # one flag serves all three outputs: dq adds from the second step on, so this block's (fresh) dk/dv
        # buffers start at zero then, and at NaN for the first step to show that they are overwritten
        dkb = torch.full((bs, b - a, hkv, hs), 0.0 if step else float("nan"), dtype=torch.float32, device="cuda")
        dvb = dkb.clone()
        usp.usp_block_attn_bwd(q, kb, vb, d_o, lse, delta, dq, dkb, dvb, bs, Lq, b - a, hq, hkv, hs, 0.0, causal, qdesc,
                               kdb, step > 0)
        dk[:, a:b] = dkb
        dv[:, a:b] = dvb
    torch.cuda.synchronize()
    for name, got, ref in (("dq", dq, ref_dq), ("dk", dk, ref_dk), ("dv", dv, ref_dv)):
        g = tl.to_f64(got)
        assert not np.isnan(g).any(), name
        assert tl.max_abs(g, ref) <= GRAD_TOL, name


def test_block_attn_bwd_accumulate_adds(usp):
    bs, L, hq, hkv, hs = 1, 256, 2, 1, 128
    qs, _ = tl.gen(5, inputs.TENSOR_Q, bs, np.arange(L), np.arange(hq), hs, tl.BF16)
    ks, _ = tl.gen(5, inputs.TENSOR_K, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    vs, _ = tl.gen(5, inputs.TENSOR_V, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    gs, _ = tl.gen(5, inputs.TENSOR_DO, bs, np.arange(L), np.arange(hq), hs, tl.BF16)
    q, k, v, d_o = (tl.to_device(x, tl.BF16) for x in (qs, ks, vs, gs))
    d = usp.usp_posdesc(0, L, 0, 0)
    o = torch.empty_like(q)
    lse = torch.empty((bs, hq, L), dtype=torch.float32, device="cuda")
    usp.usp_block_attn_fwd(q, k, v, o, lse, bs, L, L, hq, hkv, hs, 0.0, True, d, d, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, L, hq, hs)
    outs = []
    for acc in (False, True):
        dq = torch.ones((bs, L, hq, hs), dtype=torch.float32, device="cuda")
        dk = torch.ones((bs, L, hkv, hs), dtype=torch.float32, device="cuda")
        dv = torch.ones((bs, L, hkv, hs), dtype=torch.float32, device="cuda")
        usp.usp_block_attn_bwd(q, k, v, d_o, lse, delta, dq, dk, dv, bs, L, L, hq, hkv, hs, 0.0, True, d, d, acc)
        torch.cuda.synchronize()
        outs.append((dq.cpu(), dk.cpu(), dv.cpu()))
    for a, b in zip(*outs):
        # same kernels on the same data; only the fp32 rounding of (1 + x) and the order of the atomic adds differ
        assert torch.allclose(a + 1.0, b, rtol=0, atol=2e-5)
    with pytest.raises(usp.UspError):
        usp.usp_block_attn_bwd(q, k, v, d_o, lse, delta, None, dk, dv, bs, L, L, hq, hkv, hs, 0.0, True, d, d, False)
    with pytest.raises(usp.UspError):
        usp.usp_block_attn_bwd(q, k, v, d_o, lse, delta, dq, dk, dv, bs, L, L, 3, 2, hs, 0.0, True, d, d, False)


def _bwd_workspace(usp, p, n_ranks, keep_ds):
    """The backward workspace, every byte 0xFF (bf16 and fp32 NaNs: a read of something never written shows); with
    keep_ds of the size at which the dK/dV kernel stores dS for the dQ kernel."""
    nb = usp.usp_attn_bwd_workspace_bytes(p, n_ranks)
    nb_ds = usp.usp_attn_bwd_workspace_bytes_with_ds(p, n_ranks)
    assert 0 < nb and (nb < nb_ds if p.hs >= 128 else nb == nb_ds)   # dS is kept at head size 128 only
    return torch.full((nb_ds if keep_ds else nb,), 0xFF, dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("keep_ds", [False, True], ids=["recompute", "stored_ds"])
@pytest.mark.parametrize("U,R,zigzag", [(2, 2, True), (1, 4, True), (4, 1, True), (2, 2, False)])
def test_usp_bwd_all_ranks(usp, U, R, zigzag, keep_ds):
    """dQ, dK, dV of every virtual rank against the textbook gradient of the unsplit Eq. 1."""
    prob = tl.Problem(91, 1, 1024, 8, 4, 128, U, R, True, zigzag, tl.BF16, with_do=True)
    p = usp.problem(prob.bs, prob.L, prob.hc, prob.hk, prob.hs, U, R, True,
                    usp.USP_SPLIT_ZIGZAG if zigzag else usp.USP_SPLIT_CONTIG, usp.USP_BF16)
    q, k, v, d_o = (prob.seq_layout_dev(n) for n in ("q", "k", "v", "do"))
    o = torch.empty_like(q)
    lse = torch.empty((prob.N, prob.bs, prob.hc // U, prob.L // R), dtype=torch.float32, device="cuda")
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
    ws2 = _bwd_workspace(usp, p, prob.N, keep_ds)
    dq = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    dk = torch.full(k.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    dv = torch.full(v.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, 0, prob.N, ws2)
    torch.cuda.synchronize()
    ref_dq, ref_dk, ref_dv = orc.attention_backward(prob.val["q"], prob.val["k"], prob.val["v"], prob.val["do"], True)
    for name, got, ref in (("dq", dq, ref_dq), ("dk", dk, ref_dk), ("dv", dv, ref_dv)):
        g = tl.to_f64(got)
        assert not np.isnan(g).any(), name
        for rank in range(prob.N):
            assert tl.max_abs(g[rank], ref[:, prob.rank_positions(rank)]) <= GRAD_TOL, (name, rank)


@pytest.mark.parametrize("name,bs,L,hc,hk,hs,U,R,causal", [
    ("mqa_ring_only", 1, 512, 4, 1, 128, 1, 4, True),
    ("head_size_64_batch2", 2, 512, 8, 4, 64, 2, 2, True),
    ("noncausal", 1, 768, 8, 4, 128, 2, 2, False),
    # more ring blocks than one launch pair takes: two pairs, the second adds to dQ
    ("ring_of_20_two_launch_pairs", 1, 2560, 4, 2, 128, 1, 20, True),
    # short sequences: dQ items in slices of their key tiles, dK/dV items in slices of their query tiles, every
    # slice with its own copy of the output (4 + 4 slices, 4 head splits; then 2 ring blocks, batch of two)
    ("sliced_items_one_block", 1, 4096, 8, 2, 128, 2, 1, True),
    ("sliced_items_two_blocks_batch_of_two", 2, 4096, 4, 2, 128, 1, 2, True),
    ("sliced_items_noncausal_hs64", 1, 3072, 4, 4, 64, 2, 1, False),
    # lengths that are no multiple of the 32-row blocks: a ragged last tile, and zigzag runs of 250 rows that
    # begin and end inside blocks
    ("ragged_length_one_rank", 1, 1000, 4, 2, 128, 1, 1, True),
    ("ragged_zigzag_runs_hs64", 1, 1000, 4, 2, 64, 1, 2, True),
    ("ragged_noncausal_two_blocks", 2, 600, 2, 1, 128, 1, 2, False),
])
@pytest.mark.parametrize("keep_ds", [False, True], ids=["recompute", "stored_ds"])
def test_usp_bwd_other_model_shapes(usp, name, bs, L, hc, hk, hs, U, R, causal, keep_ds):
    prob = tl.Problem(400 + len(name), bs, L, hc, hk, hs, U, R, causal, True, tl.BF16, with_do=True)
    p = usp.problem(bs, L, hc, hk, hs, U, R, causal, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    q, k, v, d_o = (prob.seq_layout_dev(n) for n in ("q", "k", "v", "do"))
    o = torch.empty_like(q)
    lse = torch.empty((prob.N, bs, hc // U, L // R), dtype=torch.float32, device="cuda")
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
    ws2 = _bwd_workspace(usp, p, prob.N, keep_ds)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, 0, prob.N, ws2)
    torch.cuda.synchronize()
    ref = orc.attention_backward(prob.val["q"], prob.val["k"], prob.val["v"], prob.val["do"], causal)
    for name_, got, r in zip(("dq", "dk", "dv"), (dq, dk, dv), ref):
        g = tl.to_f64(got)
        assert not np.isnan(g).any(), name_
        for rank in range(prob.N):
            assert tl.max_abs(g[rank], r[:, prob.rank_positions(rank)]) <= GRAD_TOL, (name_, rank)


@pytest.mark.parametrize("keep_ds", [False, True], ids=["recompute", "stored_ds"])
def test_usp_bwd_rank_range_straddling_ring_rows(usp, keep_ds):
    """Ranks [U-1, U+1) = (ring row 0, column U-1) and (ring row 1, column 0): the columns in between are not
    visited.  The visited columns' head slices of dk / dv hold the two ranks' contributions (the oracle's gradient
    restricted to each rank's query rows and heads); every other head slice of dq / dk / dv is left untouched."""
    bs, L, hc, hk, hs, U, R = 1, 1024, 8, 4, 128, 4, 2
    prob = tl.Problem(97, bs, L, hc, hk, hs, U, R, True, True, tl.BF16, with_do=True)
    p = usp.problem(bs, L, hc, hk, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    q, k, v, d_o = (prob.seq_layout_dev(n) for n in ("q", "k", "v", "do"))
    o = torch.empty_like(q)
    lse = torch.empty((prob.N, bs, hc // U, L // R), dtype=torch.float32, device="cuda")
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
    ws2 = _bwd_workspace(usp, p, 2, keep_ds)
    SENT = 768.0                                          # exactly representable in bf16
    dq = torch.full(q.shape, SENT, dtype=torch.bfloat16, device="cuda")
    dk = torch.full(k.shape, SENT, dtype=torch.bfloat16, device="cuda")
    dv = torch.full(v.shape, SENT, dtype=torch.bfloat16, device="cuda")
    usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, U - 1, U + 1, ws2)
    torch.cuda.synchronize()
    gq, gk, gv = tl.to_f64(dq), tl.to_f64(dk), tl.to_f64(dv)        # [N][bs][L/N][heads][hs]
    hq, hkv = hc // U, hk // U
    allpos = np.arange(L)
    seen_q = np.zeros(gq.shape, dtype=bool)
    seen_kv = np.zeros(gk.shape, dtype=bool)
    for rank in (U - 1, U):
        r, u = divmod(rank, U)
        rows = orc.ring_block_positions(L, R, r)
        qh, kh = slice(u * hq, (u + 1) * hq), slice(u * hkv, (u + 1) * hkv)
        rq, rk, rv = orc.attention_backward(prob.val["q"][:, rows, qh], prob.val["k"][:, :, kh], prob.val["v"][:, :, kh],
                                            prob.val["do"][:, rows, qh], True, None, rows, allpos)
        full_q = np.zeros((bs, L, hq, hs))
        full_q[:, rows] = rq
        for shard in range(prob.N):
            pos = prob.rank_positions(shard)
            if shard // U == r:                           # dQ goes to the shards of the rank's own ring row
                assert tl.max_abs(gq[shard][:, :, qh], full_q[:, pos]) <= GRAD_TOL, ("dq", rank, shard)
                seen_q[shard][:, :, qh] = True
            assert tl.max_abs(gk[shard][:, :, kh], rk[:, pos]) <= GRAD_TOL, ("dk", rank, shard)
            assert tl.max_abs(gv[shard][:, :, kh], rv[:, pos]) <= GRAD_TOL, ("dv", rank, shard)
            seen_kv[shard][:, :, kh] = True
    assert (~seen_q).any() and (~seen_kv).any()
    assert np.all(gq[~seen_q] == SENT), "dq written outside the head slices of the ranks in range"
    assert np.all(gk[~seen_kv] == SENT), "dk written for a column no rank in range visited"
    assert np.all(gv[~seen_kv] == SENT), "dv written for a column no rank in range visited"


def test_usp_bwd_rejects_bad_arguments(usp):
    p32 = usp.problem(1, 256, 4, 4, 64, 2, 2, False, dtype=usp.USP_FP32)
    assert usp.usp_attn_bwd_workspace_bytes(p32, 1) == 0          # bf16 only
    p = usp.problem(1, 1024, 8, 4, 128, 2, 2, True)
    x = torch.zeros(1 << 20, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(usp.UspError) as e:
        usp.usp_attn_bwd(p, x, x, x, x, x, x, x, x, x, 0, 1, x, 64)
    assert e.value.status == 5


@pytest.mark.parametrize("keep_ds", [False, True], ids=["recompute", "stored_ds"])
def test_usp_fwd_and_bwd_in_a_hip_graph(usp, keep_ds):
    """Algorithm 1 forward and backward of all ranks captured into ONE HIP graph (some thirty kernels: permutations,
    the persistent attention kernels with their item counters, merge, conversion) and replayed with eager calls and
    synchronisations between the replays: every replay must reproduce the eager result bit for bit (the forward and
    dQ are deterministic; dK/dV too, since slices and split heads write copies that are added in a fixed order)."""
    prob = tl.Problem(93, 1, 4096, 8, 4, 128, 2, 2, True, True, tl.BF16, with_do=True)
    p = usp.problem(prob.bs, prob.L, prob.hc, prob.hk, prob.hs, 2, 2, True, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    q, k, v, d_o = (prob.seq_layout_dev(n) for n in ("q", "k", "v", "do"))
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    ws2 = _bwd_workspace(usp, p, prob.N, keep_ds)

    def outputs():
        return (torch.empty_like(q), torch.empty((prob.N, 1, 4, 2048), dtype=torch.float32, device="cuda"),
                torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))

    def run(o, lse, dq, dk, dv):
        usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
        usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, 0, prob.N, ws2)
    ref = outputs()
    run(*ref)                      # eager first: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    got = outputs()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(*got)
    eager = outputs()
    for rep in range(3):
        for t in got:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(got, ref):
            assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                               b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16)), rep
        run(*eager)                # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(eager[2].view(torch.int16), ref[2].view(torch.int16)), rep
