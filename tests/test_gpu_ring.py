"""GPU parity: the whole ring loop of one rank in ONE launch (usp_ring_attn_fwd, and its backward usp_ring_attn_bwd) against the oracle's plain
attention over the concatenated blocks, and against the stepwise path (one usp_block_attn_fwd per block, then
usp_lse_merge), through the C ABI.  Tolerances as for the block kernel: O 2e-2, LSE 1e-3 (max-abs)."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2405_07719_amd import inputs
from tests import usp_testlib as tl

pytestmark = pytest.mark.gpu


def _ring_case(usp, seed, bs, L, hq, hkv, hs, R, r, zigzag, causal, order):
    """Ring rank r of an R-way ring over a sequence of L positions: its queries against the R K/V blocks given
    in `order`.  Values are keyed by GLOBAL position, placement by the oracle's Algorithm-2 map."""
    qpos = orc.ring_block_positions(L, R, r, zigzag)
    _, gq = tl.gen(seed, inputs.TENSOR_Q, bs, np.arange(L), np.arange(hq), hs, tl.BF16)
    sk, gk = tl.gen(seed, inputs.TENSOR_K, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    sv, gv = tl.gen(seed, inputs.TENSOR_V, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    sq, _ = tl.gen(seed, inputs.TENSOR_Q, bs, qpos, np.arange(hq), hs, tl.BF16)
    q = tl.to_device(sq, tl.BF16)
    kb, vb, kd = [], [], []
    for s in order:
        kp = orc.ring_block_positions(L, R, s, zigzag)
        kb.append(tl.to_device(sk[:, kp], tl.BF16))
        vb.append(tl.to_device(sv[:, kp], tl.BF16))
        kd.append(_desc_of(usp, kp))
    ref_o, ref_l = orc.attention_rows(gq[:, qpos], qpos, gk, gv, causal)
    return q, kb, vb, kd, _desc_of(usp, qpos), ref_o, ref_l


def _desc_of(usp, pos):
    """Two-run descriptor of an ascending-run position list."""
    pos = np.asarray(pos)
    brk = np.nonzero(np.diff(pos) != 1)[0]
    if len(brk) == 0:
        return usp.usp_posdesc(int(pos[0]), len(pos), 0, 0)
    assert len(brk) == 1
    n0 = int(brk[0]) + 1
    return usp.usp_posdesc(int(pos[0]), n0, int(pos[n0]), len(pos) - n0)


@pytest.mark.parametrize("name,bs,L,hq,hkv,hs,R,r,zigzag,causal,order", [
    ("zigzag_r1_of_4", 1, 2048, 4, 2, 128, 4, 1, True, True, (1, 0, 3, 2)),
    ("zigzag_r0_of_4_sees_little", 1, 2048, 2, 1, 128, 4, 0, True, True, (0, 3, 2, 1)),
    ("contig_r2_of_4_empty_blocks", 1, 2048, 2, 2, 128, 4, 2, False, True, (2, 1, 0, 3)),
    ("noncausal_3_blocks_ragged", 2, 1500, 2, 1, 128, 3, 1, False, False, (1, 0, 2)),
    ("hs64_r3_of_8", 1, 2048, 4, 4, 64, 8, 3, True, True, (3, 2, 1, 0, 7, 6, 5, 4)),
    ("sixteen_blocks", 1, 4096, 2, 1, 128, 16, 9, True, True, tuple((9 - i) % 16 for i in range(16))),
])
@pytest.mark.parametrize("o_dtype", [tl.BF16, tl.FP32])
def test_ring_attn_fwd_matches_oracle_and_stepwise(usp, name, bs, L, hq, hkv, hs, R, r, zigzag, causal, order, o_dtype):
    q, kb, vb, kd, qd, ref_o, ref_l = _ring_case(usp, 77, bs, L, hq, hkv, hs, R, r, zigzag, causal, order)
    Lq = Lk = L // R
    tdt = torch.float32 if o_dtype == tl.FP32 else torch.bfloat16
    o = torch.full((bs, Lq, hq, hs), float("nan"), dtype=tdt, device="cuda")
    lse = torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kd if causal else None, o, lse, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                          qd if causal else None, tl.BF16, o_dtype)
    torch.cuda.synchronize()
    got_o, got_l = tl.to_f64(o), tl.to_f64(lse)
    assert not np.isnan(got_o).any() and not np.isnan(got_l).any()
    tl.assert_lse_close(got_l, ref_l, 1e-3)
    assert tl.max_abs(got_o, ref_o) <= 2e-2
    # the stepwise path: one launch per block with fp32 partials, then the merge
    parts = [torch.empty((bs, Lq, hq, hs), dtype=torch.float32, device="cuda") for _ in order]
    lparts = [torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda") for _ in order]
    for i in range(len(order)):
        usp.usp_block_attn_fwd(q, kb[i], vb[i], parts[i], lparts[i], bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                               qd if causal else None, kd[i] if causal else None, tl.BF16, tl.FP32)
    o2 = torch.empty_like(o)
    lse2 = torch.empty_like(lse)
    usp.usp_lse_merge(parts, lparts, o2, lse2, bs, Lq, hq, hs, tl.FP32, o_dtype)
    torch.cuda.synchronize()
    tl.assert_lse_close(got_l, tl.to_f64(lse2), 1e-4)
    assert tl.max_abs(got_o, tl.to_f64(o2)) <= 2e-2


def test_ring_attn_fwd_nothing_visible_gives_zero_and_minus_inf(usp):
    bs, Lq, hq, hkv, hs = 1, 300, 2, 1, 128
    q = torch.randn((bs, Lq, hq, hs), device="cuda").bfloat16()
    kb = [torch.randn((bs, Lq, hkv, hs), device="cuda").bfloat16() for _ in range(2)]
    vb = [torch.randn((bs, Lq, hkv, hs), device="cuda").bfloat16() for _ in range(2)]
    o = torch.full((bs, Lq, hq, hs), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda")
    qd = usp.usp_posdesc(0, Lq, 0, 0)
    kd = [usp.usp_posdesc(1000, Lq, 0, 0), usp.usp_posdesc(5000, Lq, 0, 0)]      # every key lies after every query
    usp.usp_ring_attn_fwd(q, kb, vb, kd, o, lse, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, tl.BF16, tl.BF16)
    torch.cuda.synchronize()
    assert bool((o == 0).all()) and bool(torch.isneginf(lse).all())


def test_ring_attn_fwd_rejects_bad_arguments(usp):
    x = torch.zeros(4096, device="cuda").bfloat16()
    l = torch.zeros(64, device="cuda")
    qd = usp.usp_posdesc(0, 8, 0, 0)
    with pytest.raises(usp.UspError):                       # no blocks
        usp.usp_ring_attn_fwd(x, [], [], [], x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd, tl.BF16, tl.BF16)
    with pytest.raises(usp.UspError):                       # too many blocks
        usp.usp_ring_attn_fwd(x, [x] * 17, [x] * 17, [qd] * 17, x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd, tl.BF16, tl.BF16)
    with pytest.raises(usp.UspError) as e:                  # fp32 inputs are not supported by this entry point
        usp.usp_ring_attn_fwd(x, [x], [x], [qd], x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd, tl.FP32, tl.BF16)
    assert e.value.status == 4
    with pytest.raises(usp.UspError):                       # a descriptor that does not cover Lk keys
        usp.usp_ring_attn_fwd(x, [x], [x], [usp.usp_posdesc(0, 7, 0, 0)], x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd,
                              tl.BF16, tl.BF16)
    with pytest.raises(usp.UspError):                       # causal without descriptors
        usp.usp_ring_attn_fwd(x, [x], [x], None, x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd, tl.BF16, tl.BF16)


def test_ring_attn_bwd_matches_per_block_calls(usp):
    """The ring loop's backward in one launch pair against one usp_block_attn_bwd per block (same kernels, so the
    agreement is tight: only the order of the fp32 additions into dQ and the atomics differ)."""
    bs, L, hq, hkv, hs, R, r = 1, 2048, 4, 2, 128, 4, 2
    order = (2, 1, 0, 3)
    q, kb, vb, kd, qd, _, _ = _ring_case(usp, 91, bs, L, hq, hkv, hs, R, r, True, True, order)
    Lq = L // R
    d_o = torch.randn((bs, Lq, hq, hs), device="cuda").bfloat16()
    o = torch.empty_like(q)
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kd, o, lse, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, Lq, hq, hs)
    f32 = dict(dtype=torch.float32, device="cuda")
    dq = torch.full((bs, Lq, hq, hs), float("nan"), **f32)
    dk = [torch.full((bs, Lq, hkv, hs), float("nan"), **f32) for _ in order]
    dv = [torch.full((bs, Lq, hkv, hs), float("nan"), **f32) for _ in order]
    usp.usp_ring_attn_bwd(q, kb, vb, kd, d_o, lse, delta, dq, dk, dv, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, False,
                          [False] * len(order))
    dq2 = torch.full_like(dq, float("nan"))
    # the single-block call has one flag for all three outputs: dq adds from the second block on, so the later
    # blocks' (fresh) dk/dv buffers start at zero, the first block's at NaN to show that it is overwritten
    dk2 = [torch.full_like(x, float("nan") if i == 0 else 0.0) for i, x in enumerate(dk)]
    dv2 = [torch.full_like(x, float("nan") if i == 0 else 0.0) for i, x in enumerate(dv)]
    for i in range(len(order)):
        usp.usp_block_attn_bwd(q, kb[i], vb[i], d_o, lse, delta, dq2, dk2[i], dv2[i], bs, Lq, Lq, hq, hkv, hs, 0.0, True,
                               qd, kd[i], i > 0)
    torch.cuda.synchronize()
    assert torch.allclose(dq, dq2, atol=2e-5, rtol=1e-5)
    for a, b in zip(dk + dv, dk2 + dv2):
        assert not torch.isnan(a).any()
        assert torch.allclose(a, b, atol=2e-5, rtol=1e-5)
    # a second launch that adds doubles dK/dV and dQ
    usp.usp_ring_attn_bwd(q, kb, vb, kd, d_o, lse, delta, dq, dk, dv, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, True,
                          [True] * len(order))
    torch.cuda.synchronize()
    assert torch.allclose(dq, 2 * dq2, atol=4e-5, rtol=1e-5)
    assert torch.allclose(dk[1], 2 * dk2[1], atol=4e-5, rtol=1e-5)
    with pytest.raises(usp.UspError):
        usp.usp_ring_attn_bwd(q, [], [], [], d_o, lse, delta, dq, [], [], bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, False, [])


def test_many_launches_leave_the_item_counters_clean(usp):
    """The forward kernel's workgroups draw their work items from per-launch counters that the last draw of a
    launch puts back to zero, and the launches take the counter sets in rotation: more launches than there are
    sets, of two alternating shapes (one with fewer items than CUs, one with more items than CUs and eight KV
    heads, i.e. eight item queues), must all give the first launch's result, bit for bit."""
    shapes = [(1, 300, 3, 1, 64), (2, 2500, 16, 8, 128)]   # bs, L, hq, hkv, hs -> 6 items / 320 items
    runs = []
    for bs, L, hq, hkv, hs in shapes:
        qs, _ = tl.gen(77, inputs.TENSOR_Q, bs, np.arange(L), np.arange(hq), hs, tl.BF16)
        ks, _ = tl.gen(77, inputs.TENSOR_K, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
        vs, _ = tl.gen(77, inputs.TENSOR_V, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
        q, k, v = (tl.to_device(x, tl.BF16) for x in (qs, ks, vs))
        d = usp.usp_posdesc(0, L, 0, 0)
        o = torch.empty_like(q)
        lse = torch.empty((bs, hq, L), dtype=torch.float32, device="cuda")
        runs.append((q, k, v, d, o, lse, bs, L, hq, hkv, hs))
    first = []
    for i in range(2 * 300):
        q, k, v, d, o, lse, bs, L, hq, hkv, hs = runs[i % 2]
        o.fill_(float("nan"))
        usp.usp_block_attn_fwd(q, k, v, o, lse, bs, L, L, hq, hkv, hs, 0.0, True, d, d, tl.BF16, tl.BF16)
        if i < 2:
            torch.cuda.synchronize()
            first.append((o.clone(), lse.clone()))
        elif i % 97 < 2 or i >= 2 * 300 - 2:
            torch.cuda.synchronize()
            assert torch.equal(o.view(torch.int16), first[i % 2][0].view(torch.int16)), i
            assert torch.equal(lse, first[i % 2][1]), i


def test_launches_that_overlap_on_two_streams(usp):
    """Forward launches issued alternately on two streams (default priority) may execute at the same time; each uses
    its own set of item counters, so both streams' results must equal the single-stream ones, bit for bit."""
    bs, L, hq, hkv, hs = 1, 6000, 8, 2, 128          # 24 query tiles x 8 heads = 192 items: half the chip per launch
    qs, _ = tl.gen(78, inputs.TENSOR_Q, bs, np.arange(L), np.arange(hq), hs, tl.BF16)
    ks, _ = tl.gen(78, inputs.TENSOR_K, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    vs, _ = tl.gen(78, inputs.TENSOR_V, bs, np.arange(L), np.arange(hkv), hs, tl.BF16)
    q, k, v = (tl.to_device(x, tl.BF16) for x in (qs, ks, vs))
    d = usp.usp_posdesc(0, L, 0, 0)
    ref_o = torch.empty_like(q)
    ref_l = torch.empty((bs, hq, L), dtype=torch.float32, device="cuda")
    usp.usp_block_attn_fwd(q, k, v, ref_o, ref_l, bs, L, L, hq, hkv, hs, 0.0, True, d, d, tl.BF16, tl.BF16)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [(torch.empty_like(q), torch.empty_like(ref_l)) for _ in range(2)]
    for i in range(40):
        o, lse = outs[i % 2]
        usp.usp_block_attn_fwd(q, k, v, o, lse, bs, L, L, hq, hkv, hs, 0.0, True, d, d, tl.BF16, tl.BF16,
                               stream=streams[i % 2])
    for s in streams:
        s.synchronize()
    for o, lse in outs:
        assert torch.equal(o.view(torch.int16), ref_o.view(torch.int16))
        assert torch.equal(lse, ref_l)
    # and the counters are clean afterwards
    o2 = torch.empty_like(q)
    usp.usp_block_attn_fwd(q, k, v, o2, ref_l.clone(), bs, L, L, hq, hkv, hs, 0.0, True, d, d, tl.BF16, tl.BF16)
    torch.cuda.synchronize()
    assert torch.equal(o2.view(torch.int16), ref_o.view(torch.int16))


def test_ring_attn_fwd_in_a_hip_graph(usp):
    """The one-launch ring forward captured into a HIP graph and replayed: every replay, with eager launches and
    synchronisations between the replays, must reproduce the eager result bit for bit (the kernel's item counters
    are back at zero after each run, and a captured launch keeps its set of counters)."""
    q, kb, vb, kd, qd, _, _ = _ring_case(usp, 61, 1, 4096, 8, 4, 128, 4, 1, True, True, [1, 0, 3, 2])
    bs, Lq, hq, hkv, hs = 1, 1024, 8, 4, 128
    o_ref = torch.empty_like(q)
    l_ref = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")

    def launch(o, lse):
        usp.usp_ring_attn_fwd(q, kb, vb, kd, o, lse, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, tl.BF16, tl.BF16)
    launch(o_ref, l_ref)            # eager first: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    o_g, l_g = torch.empty_like(q), torch.empty_like(l_ref)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        launch(o_g, l_g)
    o_e, l_e = torch.empty_like(q), torch.empty_like(l_ref)
    for rep in range(4):
        o_g.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_g.view(torch.int16), o_ref.view(torch.int16)), rep
        assert torch.equal(l_g, l_ref), rep
        launch(o_e, l_e)            # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(o_e.view(torch.int16), o_ref.view(torch.int16)), rep


@pytest.mark.parametrize("causal", [True, False])
def test_ring_attn_fwd_partials_of_pieces_merge_to_the_whole(usp, causal):
    """Key split: pieces of ONE K/V tensor (unequal, not tile-aligned, batch of two) as the blocks of
    usp_ring_attn_fwd_partials; the merged partials against the oracle's plain attention and against the unsplit
    launch.  A piece that a query row cannot see must come back as O = 0, LSE = -inf for that row."""
    bs, Lq, Lk, hq, hkv, hs = 2, 700, 1000, 4, 2, 128
    cuts = [0, 300, 364, 1000]
    qpos = np.arange(250, 250 + Lq)          # rows 250..949: the first rows see nothing of the last piece
    kpos = np.arange(Lk)
    sq, gq = tl.gen(91, inputs.TENSOR_Q, bs, qpos, np.arange(hq), hs, tl.BF16)
    sk, gk = tl.gen(91, inputs.TENSOR_K, bs, kpos, np.arange(hkv), hs, tl.BF16)
    sv, gv = tl.gen(91, inputs.TENSOR_V, bs, kpos, np.arange(hkv), hs, tl.BF16)
    ref_o, ref_l = orc.block_attention(gq, gk, gv, qpos, kpos, causal)
    q, k, v = (tl.to_device(x, tl.BF16) for x in (sq, sk, sv))
    qd = usp.usp_posdesc(250, Lq, 0, 0)
    row = hkv * hs * 2
    n = len(cuts) - 1
    kb = [k.data_ptr() + a * row for a in cuts[:-1]]
    vb = [v.data_ptr() + a * row for a in cuts[:-1]]
    lk = [b - a for a, b in zip(cuts, cuts[1:])]
    kd = [usp.usp_posdesc(a, b - a, 0, 0) for a, b in zip(cuts, cuts[1:])]
    o_parts = [torch.full((bs, Lq, hq, hs), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n)]
    l_parts = [torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n)]
    usp.usp_ring_attn_fwd_partials(q, kb, vb, kd if causal else None, lk, o_parts, l_parts, bs, Lq, Lk, hq, hkv, hs,
                                   0.0, causal, qd if causal else None)
    o = torch.empty((bs, Lq, hq, hs), dtype=torch.float32, device="cuda")
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_lse_merge(o_parts, l_parts, o, lse, bs, Lq, hq, hs, tl.FP32, tl.FP32)
    o1 = torch.empty_like(o)
    l1 = torch.empty_like(lse)
    usp.usp_ring_attn_fwd(q, [k], [v], [usp.usp_posdesc(0, Lk, 0, 0)], o1, l1, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                          qd, tl.BF16, tl.FP32)
    torch.cuda.synchronize()
    for part_o, part_l in zip(o_parts, l_parts):
        assert not torch.isnan(part_o).any() and not torch.isnan(part_l).any()
    tl.assert_lse_close(tl.to_f64(lse), ref_l, 1e-3)
    assert tl.max_abs(tl.to_f64(o), ref_o) <= 2e-2
    assert tl.max_abs(tl.to_f64(o), tl.to_f64(o1)) <= 1e-2
    if causal:   # rows at positions below 364 see nothing of the last piece
        dead = int(364 - 250)
        assert torch.isneginf(l_parts[2][:, :, :dead]).all() and (o_parts[2][:, :dead] == 0).all()
        assert torch.isfinite(l_parts[2][:, :, dead:]).all()
    with pytest.raises(usp.UspError):
        usp.usp_ring_attn_fwd_partials(q, kb, vb, kd, [300, 64, 2000], o_parts, l_parts, bs, Lq, Lk, hq, hkv, hs, 0.0,
                                       causal, qd)


@pytest.mark.parametrize("keep_ds", [False, True], ids=["recompute", "stored_ds"])
@pytest.mark.parametrize("bs,L,hq,hkv,hs,R", [
    (1, 1332, 2, 1, 128, 2),      # ragged: 666 rows per rank in zigzag runs of 333
    (1, 4096, 4, 1, 128, 2),      # 2 slices of the dQ items; 4 head splits x 4 query slices = 16 copies of dK/dV
    (2, 2048, 4, 2, 64, 4),       # batch of two, head size 64, four blocks
    (1, 16384, 16, 8, 128, 4),    # two heads per K/V head over a long block: copies of dK/dV only
    (2, 16384, 8, 8, 128, 2),     # full grids, one head per K/V head: no copies at all, the workspace size is 0
])
def test_ring_attn_bwd_ws_copies_instead_of_atomics(usp, bs, L, hq, hkv, hs, R, keep_ds):
    """usp_ring_attn_bwd_ws (slices of the work items write copies into a workspace, one pass adds them up) against
    usp_ring_attn_bwd (one copy, split heads meet through atomic adds): same gradients up to fp32 rounding order;
    the accumulate flags add to what is there; two runs of the workspace variant agree bit for bit.  With keep_ds the
    workspace has room for dS and the dK/dV kernel keeps it for the dQ kernel (workspace pre-filled with NaN bytes)."""
    r = 1
    order = [(r - i) % R for i in range(R)]
    q, kb, vb, kd, qd, _, _ = _ring_case(usp, 95, bs, L, hq, hkv, hs, R, r, True, True, order)
    Lq = L // R
    d_o = torch.randn((bs, Lq, hq, hs), device="cuda").bfloat16()
    o = torch.empty_like(q)
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kd, o, lse, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, Lq, hq, hs)
    f32 = dict(dtype=torch.float32, device="cuda")

    def fresh(fill):
        return (torch.full((bs, Lq, hq, hs), fill, **f32), [torch.full((bs, Lq, hkv, hs), fill, **f32) for _ in order],
                [torch.full((bs, Lq, hkv, hs), fill, **f32) for _ in order])
    dq0, dk0, dv0 = fresh(float("nan"))
    usp.usp_ring_attn_bwd(q, kb, vb, kd, d_o, lse, delta, dq0, dk0, dv0, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, False,
                          [False] * R)
    nbytes = usp.usp_ring_attn_bwd_workspace_bytes(bs, Lq, Lq, hq, hkv, hs, R)
    assert (nbytes == 0) == (hq == hkv)
    if keep_ds:
        n_ds = usp.usp_ring_attn_bwd_workspace_bytes_with_ds(bs, Lq, Lq, hq, hkv, hs, R)
        assert n_ds >= nbytes + bs * hq * R * Lq * Lq * 2 if hs >= 128 else n_ds == nbytes   # head size 128 only
        nbytes = n_ds
    ws = torch.full((max(nbytes, 256),), 0xFF, dtype=torch.uint8, device="cuda")
    runs = []
    for _ in range(2):
        dq1, dk1, dv1 = fresh(float("nan"))
        usp.usp_ring_attn_bwd_ws(q, kb, vb, kd, d_o, lse, delta, dq1, dk1, dv1, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd,
                                 False, [False] * R, ws, nbytes)
        runs.append((dq1, dk1, dv1))
    torch.cuda.synchronize()
    dq1, dk1, dv1 = runs[0]
    for i, (a, b) in enumerate(zip([dq1] + dk1 + dv1, [dq0] + dk0 + dv0)):
        assert not torch.isnan(a).any()
        # dq from the stored dS: P comes out of the dK/dV kernel's arithmetic there (LSE folded into the product),
        # so a dS element now and then rounds to the neighbouring bf16 value: one such step moves dq by some 1e-3
        loose = keep_ds and i == 0
        assert torch.allclose(a, b, atol=5e-3 if loose else 3e-5, rtol=1e-5), i
    for a, b in zip([runs[0][0]] + runs[0][1] + runs[0][2], [runs[1][0]] + runs[1][1] + runs[1][2]):
        assert torch.equal(a, b)
    # accumulate: dq and the blocks flagged so are added to, the others overwritten
    flags = [i % 2 == 1 for i in range(R)]
    dq2, dk2, dv2 = fresh(1.0)
    usp.usp_ring_attn_bwd_ws(q, kb, vb, kd, d_o, lse, delta, dq2, dk2, dv2, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd, True,
                             flags, ws, nbytes)
    torch.cuda.synchronize()
    assert torch.allclose(dq2, dq1 + 1.0, atol=1e-6, rtol=1e-6)
    for i in range(R):
        want_k = dk1[i] + 1.0 if flags[i] else dk1[i]
        assert torch.allclose(dk2[i], want_k, atol=1e-6, rtol=1e-6), i
    if nbytes and not keep_ds:
        with pytest.raises(usp.UspError):
            usp.usp_ring_attn_bwd_ws(q, kb, vb, kd, d_o, lse, delta, dq2, dk2, dv2, bs, Lq, Lq, hq, hkv, hs, 0.0, True, qd,
                                     False, flags, ws, nbytes - 256)


# ------------------------------------------------------------------ one block per call, running state in and out
def _run_state_ring(usp, q, kb, vb, kd, qd, bs, Lq, lks, hq, hkv, hs, causal, o_dtype, poison=True):
    """One usp_block_attn_fwd_state call per block, in the order given; returns (o, lse) of the last call."""
    n = usp.usp_block_attn_fwd_state_bytes(bs, Lq, hq, hs)
    assert n >= bs * hq * Lq * (hs + 2) * 4
    # the state starts as NaN bytes (the first call must not read it), and so do the outputs (only the last call writes)
    state = torch.full((n,), 0xFF, dtype=torch.uint8, device="cuda")
    tdt = torch.float32 if o_dtype == tl.FP32 else torch.bfloat16
    o = torch.full((bs, Lq, hq, hs), float("nan"), dtype=tdt, device="cuda")
    lse = torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda")
    for i in range(len(kb)):
        last = i == len(kb) - 1
        usp.usp_block_attn_fwd_state(q, kb[i], vb[i], state, o if last else None, lse if last else None, bs, Lq, lks[i],
                                     hq, hkv, hs, 0.0, causal, qd if causal else None, kd[i] if causal else None,
                                     i == 0, last, o_dtype)
        if not last:
            torch.cuda.synchronize()
            assert bool(torch.isnan(o.float()).all()) and bool(torch.isnan(lse).all())   # untouched before the last step
    torch.cuda.synchronize()
    return tl.to_f64(o), tl.to_f64(lse)


@pytest.mark.parametrize("name,bs,L,hq,hkv,hs,R,r,zigzag,causal,order", [
    ("zigzag_r1_of_4", 1, 2048, 4, 2, 128, 4, 1, True, True, (1, 0, 3, 2)),
    ("zigzag_r0_of_4_rows_dead_in_three_steps", 1, 2048, 2, 1, 128, 4, 0, True, True, (3, 2, 1, 0)),
    ("contig_r2_of_4_empty_blocks_first", 1, 2048, 2, 2, 128, 4, 2, False, True, (3, 2, 1, 0)),
    ("noncausal_3_blocks_ragged", 2, 1500, 2, 1, 128, 3, 1, False, False, (1, 0, 2)),
    ("hs64_r3_of_8", 1, 2048, 4, 4, 64, 8, 3, True, True, (3, 2, 1, 0, 7, 6, 5, 4)),
    ("single_block_first_and_last", 1, 512, 2, 1, 128, 1, 0, True, True, (0,)),
])
@pytest.mark.parametrize("o_dtype", [tl.BF16, tl.FP32])
def test_block_attn_fwd_state_ring_matches_oracle(usp, name, bs, L, hq, hkv, hs, R, r, zigzag, causal, order, o_dtype):
    """A ring that receives one block per step: R calls with the running state carried between them equal the
    oracle's plain attention over all keys (and the one-launch ring loop, up to rounding)."""
    q, kb, vb, kd, qd, ref_o, ref_l = _ring_case(usp, 79, bs, L, hq, hkv, hs, R, r, zigzag, causal, order)
    Lq = L // R
    got_o, got_l = _run_state_ring(usp, q, kb, vb, kd, qd, bs, Lq, [Lq] * len(order), hq, hkv, hs, causal, o_dtype)
    assert not np.isnan(got_o).any() and not np.isnan(got_l).any()
    tl.assert_lse_close(got_l, ref_l, 1e-3)
    assert tl.max_abs(got_o, ref_o) <= 2e-2
    dead = np.isneginf(ref_l)
    assert np.all(got_o[np.transpose(dead, (0, 2, 1))] == 0.0)
    o1 = torch.empty((bs, Lq, hq, hs), dtype=torch.float32 if o_dtype == tl.FP32 else torch.bfloat16, device="cuda")
    l1 = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kd if causal else None, o1, l1, bs, Lq, Lq, hq, hkv, hs, 0.0, causal,
                          qd if causal else None, tl.BF16, o_dtype)
    torch.cuda.synchronize()
    tl.assert_lse_close(got_l, tl.to_f64(l1), 1e-4)
    assert tl.max_abs(got_o, tl.to_f64(o1)) <= 1e-2


def test_block_attn_fwd_state_every_mask_case_in_key_pieces(usp):
    """Every mask case of the block kernel's tests, with the keys of the block handed over in three pieces (a ragged
    one among them): rows are dead in some pieces and live in others."""
    from tests.test_gpu_attn_fwd import BLOCK_CASES
    for case in BLOCK_CASES:
        name, bs, Lq, Lk, hq, hkv, hs, causal, qd, kd = case
        qdesc = usp.usp_posdesc(*(list(qd) + [0] * (4 - len(qd)))) if qd else None
        kdesc = usp.usp_posdesc(*(list(kd) + [0] * (4 - len(kd)))) if kd else None
        qpos = np.array(qdesc.positions()) if causal else np.arange(Lq)
        kpos = np.array(kdesc.positions()) if causal else np.arange(Lk)
        qs, qv = tl.gen(44, inputs.TENSOR_Q, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
        ks, kv = tl.gen(44, inputs.TENSOR_K, bs, np.arange(Lk), np.arange(hkv), hs, tl.BF16)
        vs, vv = tl.gen(44, inputs.TENSOR_V, bs, np.arange(Lk), np.arange(hkv), hs, tl.BF16)
        ref_o, ref_l = orc.block_attention(qv, kv, vv, qpos, kpos, causal)
        q = tl.to_device(qs, tl.BF16)
        cuts = [0, Lk // 3 + 5, (2 * Lk) // 3, Lk]
        kb, vb, kds, lks = [], [], [], []
        for a, b in zip(cuts, cuts[1:]):
            kb.append(tl.to_device(ks[:, a:b], tl.BF16))
            vb.append(tl.to_device(vs[:, a:b], tl.BF16))
            kds.append(_desc_of(usp, kpos[a:b]) if causal else None)
            lks.append(b - a)
        got_o, got_l = _run_state_ring(usp, q, kb, vb, kds, qdesc, bs, Lq, lks, hq, hkv, hs, causal, tl.FP32)
        assert not np.isnan(got_o).any() and not np.isnan(got_l).any(), name
        tl.assert_lse_close(got_l, ref_l, 1e-3)
        assert tl.max_abs(got_o, ref_o) <= 2e-2, name
        dead = np.isneginf(ref_l)
        assert np.all(got_o[np.transpose(dead, (0, 2, 1))] == 0.0), name


def test_block_attn_fwd_state_rejects_bad_arguments(usp):
    x = torch.zeros(1 << 16, device="cuda").bfloat16()
    l = torch.zeros(64, device="cuda")
    qd = usp.usp_posdesc(0, 8, 0, 0)
    state = torch.zeros(usp.usp_block_attn_fwd_state_bytes(1, 8, 1, 128), dtype=torch.uint8, device="cuda")
    assert usp.usp_block_attn_fwd_state_bytes(1, 8, 1, 96) == 0
    with pytest.raises(usp.UspError) as e:                  # state too small
        usp.usp_block_attn_fwd_state(x, x, x, state[:1024], x, l, 1, 8, 8, 1, 1, 128, 0.0, True, qd, qd, True, True, tl.BF16)
    assert e.value.status == 5
    with pytest.raises(usp.UspError):                       # last step without outputs
        usp.usp_block_attn_fwd_state(x, x, x, state, None, None, 1, 8, 8, 1, 1, 128, 0.0, True, qd, qd, True, True, tl.BF16)
    with pytest.raises(usp.UspError):                       # causal without descriptors
        usp.usp_block_attn_fwd_state(x, x, x, state, x, l, 1, 8, 8, 1, 1, 128, 0.0, True, None, None, True, True, tl.BF16)


# ------------------------------------------------------------------ V blocks in key-tile-transposed layout
@pytest.mark.parametrize("name,bs,L,hq,hkv,hs,R,r,zigzag,causal,order", [
    ("zigzag_r1_of_4", 1, 2048, 4, 2, 128, 4, 1, True, True, (1, 0, 3, 2)),
    ("noncausal_3_blocks_ragged", 2, 1500, 2, 1, 128, 3, 1, False, False, (1, 0, 2)),
    ("hs64_r3_of_8", 1, 2048, 4, 4, 64, 8, 3, True, True, (3, 2, 1, 0, 7, 6, 5, 4)),
    ("one_block_ragged_causal", 1, 1000, 4, 1, 128, 1, 0, True, True, (0,)),
])
def test_ring_attn_fwd_vt_equals_row_major_v(usp, name, bs, L, hq, hkv, hs, R, r, zigzag, causal, order):
    """The ring loop with V in key-tile-transposed layout (made by usp_layout_a2a from the same blocks): bit-equal to
    the ring loop on row-major V, and within tolerance of the oracle."""
    q, kb, vb, kd, qd, ref_o, ref_l = _ring_case(usp, 83, bs, L, hq, hkv, hs, R, r, zigzag, causal, order)
    Lq = Lk = L // R
    # a block [bs, Lk, hkv, hs] is the sequence layout of a one-rank problem: its VT form comes from the layout call
    pb = usp.problem(bs, Lk, hkv, hkv, hs, 1, 1, False, usp.USP_SPLIT_CONTIG, tl.BF16)
    tiles = (Lk + 63) // 64
    vt = []
    for v in vb:
        t = torch.full((bs, hkv, tiles, hs, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
        usp.usp_layout_a2a(pb, hkv, usp.USP_SEQ_TO_HEAD_VT, v, t, 0, 1)
        vt.append(t)
    o0 = torch.full((bs, Lq, hq, hs), float("nan"), dtype=torch.bfloat16, device="cuda")
    l0 = torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda")
    o1, l1 = o0.clone(), l0.clone()
    usp.usp_ring_attn_fwd(q, kb, vb, kd if causal else None, o0, l0, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                          qd if causal else None, tl.BF16, tl.BF16)
    usp.usp_ring_attn_fwd_vt(q, kb, vt, kd if causal else None, o1, l1, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                             qd if causal else None)
    torch.cuda.synchronize()
    assert torch.equal(o0.view(torch.int16), o1.view(torch.int16))
    assert torch.equal(l0.view(torch.int32), l1.view(torch.int32))
    tl.assert_lse_close(tl.to_f64(l1), ref_l, 1e-3)
    assert tl.max_abs(tl.to_f64(o1), ref_o) <= 2e-2
