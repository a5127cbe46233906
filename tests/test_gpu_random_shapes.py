"""GPU parity on randomly drawn shapes and position descriptors (seeded): ragged lengths, arbitrary two-run
descriptors whose runs are not aligned to any tile size and may be out of order, GQA groups, both head sizes,
one to five K/V blocks per launch; and whole problems of medium length (random U, R, heads, batch, chunk length)
through usp_attn_fwd and usp_attn_bwd.  Forward against the oracle's plain attention, backward against its gradient.
Tolerances as everywhere: O 2e-2, LSE 1e-3, gradients 5e-2 (max-abs)."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from paper_2405_07719_amd import inputs
from tests import usp_testlib as tl

pytestmark = pytest.mark.gpu


def _random_desc(rng, usp, n, span):
    """n local indices in one or two ascending runs placed anywhere in [0, span) without overlap."""
    if n == 1 or rng.random() < 0.3:
        s0 = int(rng.integers(0, span - n + 1))
        return usp.usp_posdesc(s0, n, 0, 0)
    n0 = int(rng.integers(1, n))
    n1 = n - n0
    # two disjoint intervals, in either order
    lo_len, hi_len = (n0, n1) if rng.random() < 0.5 else (n1, n0)
    lo = int(rng.integers(0, span - n + 1))
    hi = int(rng.integers(lo + lo_len, span - hi_len + 1))
    if lo_len == n0 and rng.random() < 0.7:
        return usp.usp_posdesc(lo, n0, hi, n1)          # ascending overall (the Algorithm-2 case)
    return usp.usp_posdesc(hi, hi_len, lo, lo_len) if hi_len == n0 else usp.usp_posdesc(lo, n0, hi, n1)


def _draw(rng, usp, max_len):
    hs = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 4]))
    bs = int(rng.choice([1, 2]))
    Lq = int(rng.integers(1, max_len))
    Lk = int(rng.integers(1, max_len))
    nb = int(rng.integers(1, 6))
    causal = bool(rng.random() < 0.8)
    span = 4 * max_len
    qd = _random_desc(rng, usp, Lq, span)
    kds = [_random_desc(rng, usp, Lk, span) for _ in range(nb)]
    return bs, Lq, Lk, hkv * g, hkv, hs, nb, causal, qd, kds


def _tensors(seed, bs, Lq, Lk, hq, hkv, hs, nb):
    qs, qv = tl.gen(seed, inputs.TENSOR_Q, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
    ks, kv = tl.gen(seed, inputs.TENSOR_K, bs, np.arange(nb * Lk), np.arange(hkv), hs, tl.BF16)
    vs, vv = tl.gen(seed, inputs.TENSOR_V, bs, np.arange(nb * Lk), np.arange(hkv), hs, tl.BF16)
    return qs, qv, ks, kv, vs, vv


@pytest.mark.parametrize("seed", range(24))
def test_ring_fwd_random_shapes(usp, seed):
    rng = np.random.default_rng(1000 + seed)
    _check_ring_fwd(usp, seed, _draw(rng, usp, 700))


@pytest.mark.parametrize("seed", range(8))
def test_ring_fwd_random_shapes_of_many_tiles(usp, seed):
    """The same with blocks of up to 24 key tiles: long runs of tiles that need no mask between the unaligned
    boundaries of the position runs, where the kernels decide per tile from runs worked out once per block."""
    rng = np.random.default_rng(7000 + seed)
    bs, Lq, Lk, hq, hkv, hs, nb, causal, qd, kds = _draw(rng, usp, 1500)
    Lq, Lk = max(Lq, 300), max(Lk, 700)
    span = int(1.3 * max(Lq, Lk)) + 10    # queries and keys share a narrow range of positions: boundaries everywhere
    qd = _random_desc(rng, usp, Lq, span)
    kds = [_random_desc(rng, usp, Lk, span) for _ in range(nb)]
    _check_ring_fwd(usp, 300 + seed, (1, Lq, Lk, hq, hkv, hs, min(nb, 3), True, qd, kds[:min(nb, 3)]))


def _check_ring_fwd(usp, seed, drawn):
    bs, Lq, Lk, hq, hkv, hs, nb, causal, qd, kds = drawn
    qs, qv, ks, kv, vs, vv = _tensors(seed, bs, Lq, Lk, hq, hkv, hs, nb)
    qpos = np.array(qd.positions()) if causal else np.arange(Lq)
    kpos = np.concatenate([np.array(d.positions()) for d in kds]) if causal else np.arange(nb * Lk)
    ref_o, ref_l = orc.block_attention(qv, kv, vv, qpos, kpos, causal, None)
    q = tl.to_device(qs, tl.BF16)
    kb = [tl.to_device(ks[:, j * Lk:(j + 1) * Lk], tl.BF16) for j in range(nb)]
    vb = [tl.to_device(vs[:, j * Lk:(j + 1) * Lk], tl.BF16) for j in range(nb)]
    o = torch.full((bs, Lq, hq, hs), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((bs, hq, Lq), float("nan"), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kds if causal else None, o, lse, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                          qd if causal else None, tl.BF16, tl.FP32)
    torch.cuda.synchronize()
    got_o, got_l = tl.to_f64(o), tl.to_f64(lse)
    assert not np.isnan(got_o).any() and not np.isnan(got_l).any()
    tl.assert_lse_close(got_l, ref_l, 1e-3)
    assert tl.max_abs(got_o, ref_o) <= 2e-2


@pytest.mark.parametrize("seed", range(12))
def test_ring_bwd_random_shapes(usp, seed):
    rng = np.random.default_rng(5000 + seed)
    _check_ring_bwd(usp, 100 + seed, _draw(rng, usp, 400))


@pytest.mark.parametrize("seed", range(6))
def test_ring_bwd_random_shapes_of_many_tiles(usp, seed):
    """Blocks of 16 ... 31 key tiles and 8 ... 31 query tiles of 32 (causal, one or two blocks): the backward
    kernels' runs of tiles that need no mask, between unaligned run boundaries.  Keys and queries of similar
    number, so that the gradients stay of the magnitude the 5e-2 tolerance is meant for."""
    rng = np.random.default_rng(9000 + seed)
    bs, Lq, Lk, hq, hkv, hs, nb, causal, qd, kds = _draw(rng, usp, 1000)
    Lq, Lk = int(rng.integers(256, 1000)), int(rng.integers(512, 1000))
    nb = min(nb, 2)
    span = int(1.3 * max(Lq, Lk)) + 10    # queries and keys share a narrow range of positions: boundaries everywhere
    qd = _random_desc(rng, usp, Lq, span)
    kds = [_random_desc(rng, usp, Lk, span) for _ in range(nb)]
    _check_ring_bwd(usp, 400 + seed, (1, Lq, Lk, hq, hkv, hs, nb, True, qd, kds), scale_tolerance=True)


def _check_ring_bwd(usp, seed, drawn, scale_tolerance=False):
    bs, Lq, Lk, hq, hkv, hs, nb, causal, qd, kds = drawn
    qs, qv, ks, kv, vs, vv = _tensors(seed, bs, Lq, Lk, hq, hkv, hs, nb)
    gs, gv = tl.gen(seed, inputs.TENSOR_DO, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
    qpos = np.array(qd.positions()) if causal else np.arange(Lq)
    kpos = np.concatenate([np.array(d.positions()) for d in kds]) if causal else np.arange(nb * Lk)
    ref_dq, ref_dk, ref_dv = orc.attention_backward(qv, kv, vv, gv, causal, None, qpos, kpos)
    q, d_o = tl.to_device(qs, tl.BF16), tl.to_device(gs, tl.BF16)
    kb = [tl.to_device(ks[:, j * Lk:(j + 1) * Lk], tl.BF16) for j in range(nb)]
    vb = [tl.to_device(vs[:, j * Lk:(j + 1) * Lk], tl.BF16) for j in range(nb)]
    o = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kds if causal else None, o, lse, bs, Lq, Lk, hq, hkv, hs, 0.0, causal,
                          qd if causal else None, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, Lq, hq, hs)
    f32 = dict(dtype=torch.float32, device="cuda")
    dq = torch.full((bs, Lq, hq, hs), float("nan"), **f32)
    dk = [torch.full((bs, Lk, hkv, hs), float("nan"), **f32) for _ in range(nb)]
    dv = [torch.full((bs, Lk, hkv, hs), float("nan"), **f32) for _ in range(nb)]
    usp.usp_ring_attn_bwd(q, kb, vb, kds if causal else None, d_o, lse, delta, dq, dk, dv, bs, Lq, Lk, hq, hkv, hs, 0.0,
                          causal, qd if causal else None, False, [False] * nb)
    torch.cuda.synchronize()
    got_dk = np.concatenate([tl.to_f64(x) for x in dk], axis=1)
    got_dv = np.concatenate([tl.to_f64(x) for x in dv], axis=1)
    for name, got, ref in (("dq", tl.to_f64(dq), ref_dq), ("dk", got_dk, ref_dk), ("dv", got_dv, ref_dv)):
        assert not np.isnan(got).any(), name
        # 5e-2 is the bound for gradients of the usual magnitude (a few units).  Random descriptors can leave hundreds of
        # queries with a handful of visible keys, whose dK / dV then reach 20-40: rounding P and dS to bf16 (2^-9
        # relative, what the kernels' matrix products take) alone moves such sums by more than 5e-2, so where asked
        # the bound grows with the reference's magnitude beyond 8.
        tol = 5e-2 * max(1.0, float(np.abs(ref).max()) / 8.0) if scale_tolerance else 5e-2
        assert tl.max_abs(got, ref) <= tol, name


@pytest.mark.parametrize("gain", [8.0, 0.015625])
def test_ring_fwd_bwd_extreme_logit_scales(usp, gain):
    """Logits with a standard deviation of ~64 (sharp softmax, exp of the raw scores would overflow) and of ~2e-4
    (flat softmax): the running-maximum handling and the statistics of the backward must hold up.  K is scaled by an
    exact power of two, so the bf16 inputs stay exact."""
    bs, Lq, Lk, hq, hkv, hs, nb = 1, 520, 384, 4, 2, 128, 3
    qs, qv, ks, kv, vs, vv = _tensors(9, bs, Lq, Lk, hq, hkv, hs, nb)
    gs, gv = tl.gen(9, inputs.TENSOR_DO, bs, np.arange(Lq), np.arange(hq), hs, tl.BF16)
    scale_q = gain * 8.0 if gain > 1 else 1.0
    qv, kv = qv * scale_q, kv * gain
    q = (tl.to_device(qs, tl.BF16).float() * scale_q).bfloat16()
    k_all = (tl.to_device(ks, tl.BF16).float() * gain).bfloat16()
    d_o = tl.to_device(gs, tl.BF16)
    qd = usp.usp_posdesc(700, Lq, 0, 0)
    kds = [usp.usp_posdesc(j * Lk, Lk, 0, 0) for j in range(nb)]
    qpos = np.array(qd.positions())
    kpos = np.concatenate([np.array(d.positions()) for d in kds])
    ref_o, ref_l = orc.block_attention(qv, kv, vv, qpos, kpos, True, None)
    ref_dq, ref_dk, ref_dv = orc.attention_backward(qv, kv, vv, gv, True, None, qpos, kpos)
    kb = [k_all[:, j * Lk:(j + 1) * Lk].contiguous() for j in range(nb)]
    vb = [tl.to_device(vs[:, j * Lk:(j + 1) * Lk], tl.BF16) for j in range(nb)]
    o = torch.empty((bs, Lq, hq, hs), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_ring_attn_fwd(q, kb, vb, kds, o, lse, bs, Lq, Lk, hq, hkv, hs, 0.0, True, qd, tl.BF16, tl.BF16)
    delta = torch.empty_like(lse)
    usp.usp_attn_delta(o, d_o, delta, bs, Lq, hq, hs)
    f32 = dict(dtype=torch.float32, device="cuda")
    dq = torch.full((bs, Lq, hq, hs), float("nan"), **f32)
    dk = [torch.full((bs, Lk, hkv, hs), float("nan"), **f32) for _ in range(nb)]
    dv = [torch.full((bs, Lk, hkv, hs), float("nan"), **f32) for _ in range(nb)]
    usp.usp_ring_attn_bwd(q, kb, vb, kds, d_o, lse, delta, dq, dk, dv, bs, Lq, Lk, hq, hkv, hs, 0.0, True, qd, False,
                          [False] * nb)
    torch.cuda.synchronize()
    tl.assert_lse_close(tl.to_f64(lse), ref_l, 1e-3 * max(1.0, float(np.max(np.abs(ref_l[np.isfinite(ref_l)]))) / 16))
    assert tl.max_abs(tl.to_f64(o), ref_o) <= 2e-2
    got_dk = np.concatenate([tl.to_f64(x) for x in dk], axis=1)
    got_dv = np.concatenate([tl.to_f64(x) for x in dv], axis=1)
    # gradients scale with the inputs' magnitudes: tolerance relative to the largest reference entry
    for name, got, ref in (("dq", tl.to_f64(dq), ref_dq), ("dk", got_dk, ref_dk), ("dv", got_dv, ref_dv)):
        assert not np.isnan(got).any(), name
        assert tl.max_abs(got, ref) <= 5e-2 * max(1.0, float(np.max(np.abs(ref)))), name


def _draw_problem(rng):
    """A whole USP problem of medium length: long enough that usp_attn_fwd cuts the keys into parts and usp_attn_bwd
    cuts its work items into slices (how, depends on every one of these numbers), small enough for the oracle."""
    while True:
        N = int(rng.choice([1, 2, 4, 8]))
        U = int(rng.choice([u for u in (1, 2, 4, 8) if N % u == 0]))
        R = N // U
        hkv_local = int(rng.choice([1, 2]))
        g = int(rng.choice([1, 2, 4]))
        hk, hc = hkv_local * U, hkv_local * U * g
        bs = int(rng.choice([1, 2]))
        hs = int(rng.choice([64, 128]))
        c = int(rng.integers(1, 40)) * 64 + int(rng.choice([0, 0, 8, 32]))     # chunk length, not always a tile multiple
        L = 2 * N * c
        if 2048 <= L <= 8192 and bs * hc * L * L <= 1.4e8:
            return bs, L, hc, hk, hs, U, R, bool(rng.random() < 0.8), bool(rng.random() < 0.75)


@pytest.mark.parametrize("seed", range(8))
def test_usp_fwd_bwd_random_problems(usp, seed):
    rng = np.random.default_rng(7000 + seed)
    bs, L, hc, hk, hs, U, R, causal, zigzag = _draw_problem(rng)
    prob = tl.Problem(7000 + seed, bs, L, hc, hk, hs, U, R, causal, zigzag, tl.BF16, with_do=True)
    p = usp.problem(bs, L, hc, hk, hs, U, R, causal, usp.USP_SPLIT_ZIGZAG if zigzag else usp.USP_SPLIT_CONTIG, usp.USP_BF16)
    q, k, v, d_o = (prob.seq_layout_dev(n) for n in ("q", "k", "v", "do"))
    o = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    lse = torch.full((prob.N, bs, hc // U, L // R), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
    ws2 = torch.empty(usp.usp_attn_bwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
    dq = torch.full(q.shape, float("nan"), dtype=q.dtype, device="cuda")
    dk = torch.full(k.shape, float("nan"), dtype=k.dtype, device="cuda")
    dv = torch.full(v.shape, float("nan"), dtype=v.dtype, device="cuda")
    usp.usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, 0, prob.N, ws2)
    torch.cuda.synchronize()
    what = (bs, L, hc, hk, hs, U, R, causal, zigzag)
    ref_o, ref_l = orc.usp_attention_reference_by_rank(prob.val["q"], prob.val["k"], prob.val["v"], causal, R, U, zigzag)
    og, lg = tl.to_f64(o), tl.to_f64(lse)
    for rank in range(prob.N):
        tl.assert_lse_close(lg[rank], ref_l[rank], 1e-3)
        assert tl.max_abs(og[rank], ref_o[rank]) <= 2e-2, (what, rank)
    refs = orc.attention_backward(prob.val["q"], prob.val["k"], prob.val["v"], prob.val["do"], causal)
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), refs):
        gg = tl.to_f64(got)
        assert not np.isnan(gg).any(), (what, name)
        for rank in range(prob.N):
            pos = orc.zigzag_positions(L, R, U, rank // U, rank % U, zigzag)
            assert tl.max_abs(gg[rank], ref[:, pos]) <= 5e-2, (what, name, rank)


@pytest.mark.parametrize("seed", range(8))
def test_usp_fwd_random_medium_problems_sampled_rows(usp, seed):
    """One rank of a randomly drawn problem of 64 ... 1024 work items (query tiles x heads x batch), causal or not,
    lengths that are no multiple of the tile sizes: where usp_attn_fwd cuts some or all query tiles into pieces of the
    keys (partial results, merged) or leaves the launch whole.  Sampled rows against the oracle's plain attention."""
    rng = np.random.default_rng(9000 + seed)
    while True:
        U = int(rng.choice([1, 2, 4, 8]))
        R = int(rng.choice([1, 1, 1, 2, 4]))
        hk = U * int(rng.choice([1, 2]))
        hc = hk * int(rng.choice([1, 2, 4]))
        hs = int(rng.choice([64, 128]))
        bs = int(rng.choice([1, 1, 2]))
        causal = bool(rng.random() < 0.6)
        tiles = max(8, int(rng.integers(64, 1024)) // (hc // U * bs))
        L = (tiles * 256 - int(rng.choice([0, 0, 64, 200]))) * R
        if L % (2 * U * R) == 0 and L <= 70000 and L * hc * bs <= 3_000_000:
            break
    rank = int(rng.integers(0, U * R))
    case = tl.OneRankCase(usp, 9000 + seed, bs, L, hc, hk, hs, U, R, rank)
    case.p = usp.problem(bs, L, hc, hk, hs, U, R, causal, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    case.forward()
    rows = case.sample_rows(rng, 48)
    pos, allpos = case.block_pos[rows], np.arange(L)
    ref_o, ref_l = orc.attention_rows(case.values(inputs.TENSOR_Q, pos, case.q_heads), pos,
                                      case.values(inputs.TENSOR_K, allpos, case.kv_heads),
                                      case.values(inputs.TENSOR_V, allpos, case.kv_heads), causal)
    got_o = case.seq_rows(case.o, rows, slice(case.u * case.hq, (case.u + 1) * case.hq))
    got_l = case.lse[case.rank].cpu().double().numpy()[:, :, rows]
    assert tl.max_abs(got_l, ref_l) <= 1e-3
    assert tl.max_abs(got_o, ref_o) <= 2e-2
