"""Pins for the CPU oracle: it is checked against things other than itself.

Brute-force loops, closed forms, invariants, library routines on the special cases
they cover, finite differences, and the one worked example the paper prints.
"""
import math
import os

import numpy as np
import pytest

from oracle import usp_oracle as orc

RNG = np.random.default_rng(7)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ brute force
def brute_attention(q, k, v, qpos, kpos, causal, scale):
    """Triple loop, math.exp only, no NumPy reductions."""
    bs, nq, hq, hs = q.shape
    nk, hkv = k.shape[1], k.shape[2]
    g = hq // hkv
    o = np.zeros((bs, nq, hq, hs))
    lse = np.full((bs, hq, nq), -np.inf)
    for b in range(bs):
        for h in range(hq):
            for i in range(nq):
                scores = []
                for j in range(nk):
                    if causal and kpos[j] > qpos[i]:
                        continue
                    s = 0.0
                    for e in range(hs):
                        s += q[b, i, h, e] * k[b, j, h // g, e]
                    scores.append((j, s * scale))
                if not scores:
                    continue
                mx = max(s for _, s in scores)
                den = sum(math.exp(s - mx) for _, s in scores)
                lse[b, h, i] = mx + math.log(den)
                for j, s in scores:
                    w = math.exp(s - mx) / den
                    for e in range(hs):
                        o[b, i, h, e] += w * v[b, j, h // g, e]
    return o, lse


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (4, 1)])
def test_attention_matches_brute_force(causal, hq, hkv):
    bs, L, hs = 2, 11, 5
    q = RNG.standard_normal((bs, L, hq, hs))
    k = RNG.standard_normal((bs, L, hkv, hs))
    v = RNG.standard_normal((bs, L, hkv, hs))
    o, lse = orc.attention(q, k, v, causal, scale=0.37)
    pos = np.arange(L)
    ob, lb = brute_attention(q, k, v, pos, pos, causal, 0.37)
    np.testing.assert_allclose(o, ob, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lb, rtol=0, atol=1e-13)


def test_block_attention_positions_match_brute_force():
    # scrambled positions, keys a strict subset, some rows see no key at all
    bs, hq, hkv, hs = 1, 4, 2, 3
    qpos = np.array([9, 0, 4, 4, 15, 2])
    kpos = np.array([3, 12, 4, 7, 1])
    q = RNG.standard_normal((bs, qpos.size, hq, hs))
    k = RNG.standard_normal((bs, kpos.size, hkv, hs))
    v = RNG.standard_normal((bs, kpos.size, hkv, hs))
    o, lse = orc.block_attention(q, k, v, qpos, kpos, True, scale=0.5)
    ob, lb = brute_attention(q, k, v, qpos, kpos, True, 0.5)
    np.testing.assert_allclose(o, ob, atol=1e-13)
    assert np.array_equal(np.isneginf(lse), np.isneginf(lb))
    fin = np.isfinite(lb)
    np.testing.assert_allclose(lse[fin], lb[fin], atol=1e-13)
    # query at position 0 sees no key (smallest key position is 1): exact zeros and -inf
    assert np.all(o[:, 1] == 0.0) and np.all(np.isneginf(lse[:, :, 1]))


def test_default_scale_is_inverse_sqrt_head_size():
    q = RNG.standard_normal((1, 6, 2, 16))
    k = RNG.standard_normal((1, 6, 2, 16))
    v = RNG.standard_normal((1, 6, 2, 16))
    o0, l0 = orc.attention(q, k, v, True)
    o1, l1 = orc.attention(q, k, v, True, scale=0.25)
    np.testing.assert_array_equal(o0, o1)
    np.testing.assert_array_equal(l0, l1)


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("causal", [False, True])
def test_zero_queries_give_running_mean_and_log_count(causal):
    bs, L, hc, hk, hs = 1, 24, 4, 2, 8
    q = np.zeros((bs, L, hc, hs))
    k = RNG.standard_normal((bs, L, hk, hs))
    v = RNG.standard_normal((bs, L, hk, hs))
    o, lse = orc.attention(q, k, v, causal)
    for p in range(L):
        n = p + 1 if causal else L
        np.testing.assert_allclose(lse[0, :, p], math.log(n), atol=1e-14)
        for h in range(hc):
            np.testing.assert_allclose(o[0, p, h], v[0, :n, h // 2].mean(axis=0), atol=1e-14)


def test_constant_values_are_returned_exactly():
    q = RNG.standard_normal((1, 9, 2, 4)) * 3
    k = RNG.standard_normal((1, 9, 2, 4)) * 3
    c = np.array([1.5, -2.0, 0.25, 7.0])
    v = np.broadcast_to(c, (1, 9, 2, 4)).copy()
    o, _ = orc.attention(q, k, v, True)
    np.testing.assert_allclose(o, v, atol=1e-14)


def test_single_visible_key():
    q = RNG.standard_normal((1, 5, 2, 4))
    k = RNG.standard_normal((1, 5, 2, 4))
    v = RNG.standard_normal((1, 5, 2, 4))
    o, lse = orc.attention(q, k, v, True, scale=0.5)
    np.testing.assert_allclose(o[0, 0], v[0, 0], atol=1e-15)
    np.testing.assert_allclose(lse[0, :, 0], 0.5 * np.einsum("he,he->h", q[0, 0], k[0, 0]), atol=1e-14)


def test_softmax_weights_sum_to_one():
    # O of the value tensor "one-hot of key index" is the weight vector itself
    L, hs = 13, 13
    q = RNG.standard_normal((1, L, 1, hs))
    k = RNG.standard_normal((1, L, 1, hs))
    v = np.eye(L)[None, :, None, :]
    o, lse = orc.attention(q, k, v, True)
    w = o[0, :, 0, :]                        # w[i, j] = weight of key j for query i
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(np.triu(w, 1) == 0.0)      # future keys carry exactly zero weight
    s = (q[0, :, 0] @ k[0, :, 0].T) / math.sqrt(hs)
    np.testing.assert_allclose(w[5, :6], np.exp(s[5, :6] - lse[0, 0, 5]), atol=1e-14)


# ------------------------------------------------------------------ library routine
@pytest.mark.parametrize("causal", [False, True])
def test_against_torch_sdpa_fp64(causal):
    torch = pytest.importorskip("torch")
    bs, L, hc, hk, hs = 2, 33, 4, 2, 16
    q = RNG.standard_normal((bs, L, hc, hs))
    k = RNG.standard_normal((bs, L, hk, hs))
    v = RNG.standard_normal((bs, L, hk, hs))
    o, _ = orc.attention(q, k, v, causal)
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(np.repeat(k, hc // hk, axis=2)).permute(0, 2, 1, 3)
    tv = torch.from_numpy(np.repeat(v, hc // hk, axis=2)).permute(0, 2, 1, 3)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)


def test_lse_against_scipy_logsumexp():
    sp = pytest.importorskip("scipy.special")
    L, hs = 10, 6
    q = RNG.standard_normal((1, L, 1, hs))
    k = RNG.standard_normal((1, L, 1, hs))
    v = RNG.standard_normal((1, L, 1, hs))
    _, lse = orc.attention(q, k, v, False, scale=0.3)
    s = 0.3 * q[0, :, 0] @ k[0, :, 0].T
    np.testing.assert_allclose(lse[0, 0], sp.logsumexp(s, axis=1), atol=1e-13)


# ------------------------------------------------------------------ backward
def _loss(q, k, v, d_o, causal, scale):
    o, _ = orc.attention(q, k, v, causal, scale)
    return float((o * d_o).sum())


@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_central_differences(causal):
    bs, L, hc, hk, hs = 1, 7, 4, 2, 3
    q = RNG.standard_normal((bs, L, hc, hs))
    k = RNG.standard_normal((bs, L, hk, hs))
    v = RNG.standard_normal((bs, L, hk, hs))
    d_o = RNG.standard_normal((bs, L, hc, hs))
    dq, dk, dv = orc.attention_backward(q, k, v, d_o, causal, scale=0.6)
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = _loss(q, k, v, d_o, causal, 0.6)
            x[idx] = old - eps
            lm = _loss(q, k, v, d_o, causal, 0.6)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=1e-6, atol=1e-8, err_msg=name)


def test_backward_constant_values_give_zero_dq_dk():
    q = RNG.standard_normal((1, 6, 2, 4))
    k = RNG.standard_normal((1, 6, 2, 4))
    v = np.broadcast_to(np.array([1.0, 2.0, 3.0, 4.0]), (1, 6, 2, 4)).copy()
    d_o = RNG.standard_normal((1, 6, 2, 4))
    dq, dk, dv = orc.attention_backward(q, k, v, d_o, True)
    np.testing.assert_allclose(dq, 0.0, atol=1e-14)
    np.testing.assert_allclose(dk, 0.0, atol=1e-14)
    # dV_j = sum_i P_ij dO_i: column sums of P weight dO; total over keys equals sum of dO rows
    np.testing.assert_allclose(dv.sum(axis=1), d_o.sum(axis=1), atol=1e-13)


def test_backward_against_torch_autograd():
    torch = pytest.importorskip("torch")
    bs, L, hc, hk, hs = 1, 12, 4, 2, 8
    q = RNG.standard_normal((bs, L, hc, hs))
    k = RNG.standard_normal((bs, L, hk, hs))
    v = RNG.standard_normal((bs, L, hk, hs))
    d_o = RNG.standard_normal((bs, L, hc, hs))
    dq, dk, dv = orc.attention_backward(q, k, v, d_o, True)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (q, k, v))
    kk = tk.repeat_interleave(hc // hk, dim=2)
    vv = tv.repeat_interleave(hc // hk, dim=2)
    o = torch.nn.functional.scaled_dot_product_attention(tq.permute(0, 2, 1, 3), kk.permute(0, 2, 1, 3), vv.permute(0, 2, 1, 3), is_causal=True)
    (o.permute(0, 2, 1, 3) * torch.tensor(d_o)).sum().backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)


def brute_backward(q, k, v, d_o, qpos, kpos, causal, scale):
    """Gradient of sum(O * dO) for Eq. 1 by scalar loops: weights w_ij from math.exp over the visible keys,
    dV_j += w_ij dO_i, dS_ij = w_ij (dO_i.V_j - sum_j' w_ij' dO_i.V_j'), dQ_i += scale dS_ij K_j, dK_j += scale dS_ij Q_i."""
    bs, nq, hq, hs = q.shape
    nk, hkv = k.shape[1], k.shape[2]
    g = hq // hkv
    dq, dk, dv = np.zeros(q.shape), np.zeros(k.shape), np.zeros(v.shape)
    for b in range(bs):
        for h in range(hq):
            kv = h // g
            for i in range(nq):
                js = [j for j in range(nk) if not causal or kpos[j] <= qpos[i]]
                if not js:
                    continue
                sc = [scale * sum(q[b, i, h, e] * k[b, j, kv, e] for e in range(hs)) for j in js]
                mx = max(sc)
                den = sum(math.exp(s - mx) for s in sc)
                w = [math.exp(s - mx) / den for s in sc]
                dp = [sum(d_o[b, i, h, e] * v[b, j, kv, e] for e in range(hs)) for j in js]
                dbar = sum(wi * di for wi, di in zip(w, dp))
                for wi, di, j in zip(w, dp, js):
                    ds = wi * (di - dbar)
                    for e in range(hs):
                        dv[b, j, kv, e] += wi * d_o[b, i, h, e]
                        dq[b, i, h, e] += scale * ds * k[b, j, kv, e]
                        dk[b, j, kv, e] += scale * ds * q[b, i, h, e]
    return dq, dk, dv


# scrambled, non-contiguous positions: the query at position 0 sees no key (smallest key position is 1), positions
# repeat (4, 4) and the orders of queries and keys differ, so a backward that ignores or swaps qpos / kpos fails
_QPOS = np.array([9, 0, 4, 4, 15, 2, 7])
_KPOS = np.array([3, 12, 4, 7, 1, 8])


def _scrambled_case(hq=4, hkv=2, hs=3):
    rng = np.random.default_rng(23)
    q = rng.standard_normal((2, _QPOS.size, hq, hs))
    k = rng.standard_normal((2, _KPOS.size, hkv, hs))
    v = rng.standard_normal((2, _KPOS.size, hkv, hs))
    d_o = rng.standard_normal((2, _QPOS.size, hq, hs))
    return q, k, v, d_o


def test_backward_with_positions_matches_brute_force():
    q, k, v, d_o = _scrambled_case()
    dq, dk, dv = orc.attention_backward(q, k, v, d_o, True, scale=0.45, qpos=_QPOS, kpos=_KPOS)
    bq, bk, bv = brute_backward(q, k, v, d_o, _QPOS, _KPOS, True, 0.45)
    np.testing.assert_allclose(dq, bq, atol=1e-13)
    np.testing.assert_allclose(dk, bk, atol=1e-13)
    np.testing.assert_allclose(dv, bv, atol=1e-13)
    assert np.all(dq[:, 1] == 0.0)                       # the row that sees no key has a zero gradient
    # and the positions matter at all: default positions give something else
    dq0, dk0, dv0 = orc.attention_backward(q, k, v, d_o, True, scale=0.45)
    assert np.abs(dq0 - dq).max() > 1e-3 and np.abs(dk0 - dk).max() > 1e-3 and np.abs(dv0 - dv).max() > 1e-3


def test_backward_with_positions_matches_central_differences_of_block_attention():
    q, k, v, d_o = _scrambled_case(hq=2, hkv=1, hs=2)

    def loss():
        o, _ = orc.block_attention(q, k, v, _QPOS, _KPOS, True, scale=0.7)
        return float((o * d_o).sum())

    dq, dk, dv = orc.attention_backward(q, k, v, d_o, True, scale=0.7, qpos=_QPOS, kpos=_KPOS)
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = loss()
            x[idx] = old - eps
            lm = loss()
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=1e-6, atol=1e-8, err_msg=name)


@pytest.mark.parametrize("ring,ulysses", [(2, 2), (4, 1), (1, 4)])
def test_backward_of_a_rank_rows_is_its_share_of_the_full_gradient(ring, ulysses):
    # P and D are row quantities, so the gradient restricted to the query rows of one Algorithm-2 shard is that
    # rank's dQ and its contribution to dK / dV; the contributions of all ranks add up to the full gradient
    bs, L, hc, hk, hs = 1, 32, 4, 2, 4
    rng = np.random.default_rng(31)
    q = rng.standard_normal((bs, L, hc, hs))
    k = rng.standard_normal((bs, L, hk, hs))
    v = rng.standard_normal((bs, L, hk, hs))
    d_o = rng.standard_normal((bs, L, hc, hs))
    fq, fk, fv = orc.attention_backward(q, k, v, d_o, True)
    sk, sv = np.zeros_like(k), np.zeros_like(v)
    kperm = rng.permutation(L)                           # keys handed over in another order than their positions
    for r in range(ring):
        for u in range(ulysses):
            rows = orc.zigzag_positions(L, ring, ulysses, r, u)
            dq, dk, dv = orc.attention_backward(q[:, rows], k[:, kperm], v[:, kperm], d_o[:, rows], True, qpos=rows, kpos=kperm)
            np.testing.assert_allclose(dq, fq[:, rows], atol=1e-13)
            sk[:, kperm] += dk
            sv[:, kperm] += dv
    np.testing.assert_allclose(sk, fk, atol=1e-12)
    np.testing.assert_allclose(sv, fv, atol=1e-12)


def test_backward_columns_match_brute_force_and_the_full_gradient():
    # selected key columns, from a subset of the query rows, with scrambled positions and a row that sees nothing
    q, k, v, d_o = _scrambled_case()
    o, lse = orc.block_attention(q, k, v, _QPOS, _KPOS, True, scale=0.45)
    delta = np.einsum("bihe,bihe->bhi", d_o, o)
    cols = np.array([4, 0, 3])
    dk, dv = orc.attention_backward_columns(q, d_o, lse, delta, _QPOS, k[:, cols], v[:, cols], _KPOS[cols], True, scale=0.45)
    _, bk, bv = brute_backward(q, k, v, d_o, _QPOS, _KPOS, True, 0.45)
    np.testing.assert_allclose(dk, bk[:, cols], atol=1e-13)
    np.testing.assert_allclose(dv, bv[:, cols], atol=1e-13)
    # a subset of the rows gives that subset's contribution: the two halves add up to the whole
    a, b = np.array([0, 2, 5]), np.array([1, 3, 4, 6])
    parts = [orc.attention_backward_columns(q[:, r], d_o[:, r], lse[:, :, r], delta[:, :, r], _QPOS[r], k[:, cols], v[:, cols],
                                            _KPOS[cols], True, scale=0.45) for r in (a, b)]
    np.testing.assert_allclose(parts[0][0] + parts[1][0], bk[:, cols], atol=1e-13)
    np.testing.assert_allclose(parts[0][1] + parts[1][1], bv[:, cols], atol=1e-13)
    # not causal: every column sees every row
    o2, lse2 = orc.block_attention(q, k, v, _QPOS, _KPOS, False, scale=0.45)
    delta2 = np.einsum("bihe,bihe->bhi", d_o, o2)
    dk2, dv2 = orc.attention_backward_columns(q, d_o, lse2, delta2, _QPOS, k[:, cols], v[:, cols], _KPOS[cols], False, scale=0.45)
    _, fk, fv = brute_backward(q, k, v, d_o, _QPOS, _KPOS, False, 0.45)
    np.testing.assert_allclose(dk2, fk[:, cols], atol=1e-13)
    np.testing.assert_allclose(dv2, fv[:, cols], atol=1e-13)


# ------------------------------------------------------------------ Algorithm 2
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "zigzag_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split(":")
            rows.append((tuple(int(x) for x in lhs.split()), [int(x) for x in rhs.split()]))
    return rows


def test_paper_worked_zigzag_example():
    rows = _golden_rows()
    assert rows
    for (L, R, U, r, u, zz), expect in rows:
        assert orc.zigzag_positions(L, R, U, r, u, bool(zz)).tolist() == expect


@pytest.mark.parametrize("L,R,U", [(16, 4, 1), (32, 2, 4), (48, 3, 2), (64, 1, 8), (64, 8, 1)])
def test_zigzag_is_a_partition_and_balanced(L, R, U):
    seen = np.concatenate([orc.zigzag_positions(L, R, U, r, u) for r in range(R) for u in range(U)])
    assert sorted(seen.tolist()) == list(range(L))
    c = L // (2 * R)
    allpos = np.arange(L)
    for r in range(R):
        blk = orc.ring_block_positions(L, R, r)
        # ascending inside the block, and the balanced causal pair count c^2 (2R-1) + c (c+1)
        assert np.all(np.diff(blk) > 0)
        assert orc.causal_pair_count(blk, allpos) == c * c * (2 * R - 1) + c * (c + 1)


def test_even_split_imbalance_is_about_seven_on_four_gpus():
    # Sec. 3: with an even split on 4 GPUs the last GPU has nearly 7x the work of the first
    L = 4096
    allpos = np.arange(L)
    w = [orc.causal_pair_count(orc.ring_block_positions(L, 4, r, zigzag=False), allpos) for r in range(4)]
    assert 6.9 < w[3] / w[0] < 7.0


# ------------------------------------------------------------------ layout maps
@pytest.mark.parametrize("U,h", [(1, 4), (2, 4), (4, 8), (8, 8)])
def test_a2a_matches_reshape_transpose_and_inverts(U, h):
    bs, n, hs = 2, 3, 5
    shards = [RNG.integers(0, 1 << 30, size=(bs, n, h, hs)) for _ in range(U)]
    # second opinion: stack -> [U', bs, n, U, h/U, hs] -> pick u -> merge (U', n)
    stack = np.stack(shards).reshape(U, bs, n, U, h // U, hs)
    heads = []
    for u in range(U):
        y = orc.a2a_seq_to_head(shards, u)
        ref = np.transpose(stack[:, :, :, u], (1, 0, 2, 3, 4)).reshape(bs, U * n, h // U, hs)
        assert np.array_equal(y, ref)
        heads.append(y)
    back = orc.a2a_head_to_seq(heads)
    for a, b in zip(back, shards):
        assert np.array_equal(a, b)
    if U == 1:
        assert np.array_equal(heads[0], shards[0])


# ------------------------------------------------------------------ merge
def test_merge_of_key_splits_equals_unsplit_attention():
    bs, L, hq, hkv, hs = 1, 20, 4, 2, 6
    q = RNG.standard_normal((bs, L, hq, hs))
    k = RNG.standard_normal((bs, L, hkv, hs))
    v = RNG.standard_normal((bs, L, hkv, hs))
    pos = np.arange(L)
    full_o, full_l = orc.attention(q, k, v, True)
    cuts = [0, 3, 11, 20]
    parts = [orc.block_attention(q, k[:, a:b], v[:, a:b], pos, pos[a:b], True) for a, b in zip(cuts, cuts[1:])]
    # early rows see nothing of the later key blocks: those partials are (0, -inf)
    assert np.all(np.isneginf(parts[2][1][:, :, :11]))
    o, l = orc.lse_merge([p[0] for p in parts], [p[1] for p in parts])
    np.testing.assert_allclose(o, full_o, atol=1e-13)
    np.testing.assert_allclose(l, full_l, atol=1e-13)
    # order of the parts is irrelevant
    o2, l2 = orc.lse_merge([p[0] for p in parts[::-1]], [p[1] for p in parts[::-1]])
    np.testing.assert_allclose(o2, o, atol=1e-14)
    np.testing.assert_allclose(l2, l, atol=1e-14)


def test_merge_special_cases():
    a = RNG.standard_normal((1, 4, 2, 3))
    b = RNG.standard_normal((1, 4, 2, 3))
    la = RNG.standard_normal((1, 2, 4))
    o, l = orc.lse_merge([a], [la])
    np.testing.assert_array_equal(o, a)
    np.testing.assert_allclose(l, la, atol=1e-15)
    o, l = orc.lse_merge([a, b], [la, la])                  # equal weights -> mean, lse + ln 2
    np.testing.assert_allclose(o, 0.5 * (a + b), atol=1e-14)
    np.testing.assert_allclose(l, la + math.log(2.0), atol=1e-14)
    ninf = np.full_like(la, -np.inf)
    o, l = orc.lse_merge([a, b], [la, ninf])                # a -inf part is ignored
    np.testing.assert_allclose(o, a, atol=1e-15)
    np.testing.assert_allclose(l, la, atol=1e-15)
    o, l = orc.lse_merge([a, b], [ninf, ninf])              # nothing visible anywhere
    assert np.all(o == 0.0) and np.all(np.isneginf(l))


# ------------------------------------------------------------------ Algorithm 1 through the definitions
@pytest.mark.parametrize("R,U,zz", [(1, 4, True), (2, 2, True), (4, 1, True), (2, 2, False), (4, 1, False)])
def test_rankwise_reference_is_factorisation_invariant(R, U, zz):
    """Ring/Ulysses split, then blockwise attention + merge + all-to-all (all in oracle terms)
    reproduces the unsplit Eq. 1 on every rank, for every factorisation U*R = N and both splits."""
    bs, L, hc, hk, hs = 1, 32, 4, 4, 4
    q = RNG.standard_normal((bs, L, hc, hs))
    k = RNG.standard_normal((bs, L, hk, hs))
    v = RNG.standard_normal((bs, L, hk, hs))
    ref_o, ref_l = orc.usp_attention_reference_by_rank(q, k, v, True, R, U, zz)
    full_o, _ = orc.attention(q, k, v, True)
    # build every rank's shard, run Algorithm 1 literally with the oracle pieces
    pos = {(r, u): orc.zigzag_positions(L, R, U, r, u, zz) for r in range(R) for u in range(U)}
    shard = {key: (q[:, p], k[:, p], v[:, p]) for key, p in pos.items()}
    head = {}
    for r in range(R):
        for u in range(U):
            head[(r, u)] = tuple(orc.a2a_seq_to_head([shard[(r, up)][t] for up in range(U)], u) for t in range(3))
    o_head = {}
    for r in range(R):
        qp = orc.ring_block_positions(L, R, r, zz)
        for u in range(U):
            parts = []
            for i in range(R):
                s = (r - i) % R
                kp = orc.ring_block_positions(L, R, s, zz)
                parts.append(orc.block_attention(head[(r, u)][0], head[(s, u)][1], head[(s, u)][2], qp, kp, True))
            o_head[(r, u)], lse = orc.lse_merge([p[0] for p in parts], [p[1] for p in parts])
            np.testing.assert_allclose(lse, ref_l[r * U + u], atol=1e-12)
    for r in range(R):
        outs = orc.a2a_head_to_seq([o_head[(r, u)] for u in range(U)])
        for up in range(U):
            np.testing.assert_allclose(outs[up], ref_o[r * U + up], atol=1e-12)
            np.testing.assert_allclose(outs[up], full_o[:, pos[(r, up)]], atol=1e-12)


def test_zigzag_step_mask_structure():
    """Under the zigzag split a ring step (r, s) is: s == r lower-triangular on local indices;
    s < r every query sees exactly the first half of the block; s > r only the second half
    of the queries sees anything, and then the whole block.  Each off-diagonal step is 2c^2 pairs."""
    L, R = 64, 4
    c = L // (2 * R)
    for r in range(R):
        qp = orc.ring_block_positions(L, R, r)
        for s in range(R):
            kp = orc.ring_block_positions(L, R, s)
            vis = kp[None, :] <= qp[:, None]
            if s == r:
                assert np.array_equal(vis, np.tril(np.ones((2 * c, 2 * c), dtype=bool)))
            elif s < r:
                assert vis[:, :c].all() and not vis[:, c:].any()
            else:
                assert not vis[:c].any() and vis[c:].all()
            if s != r:
                assert vis.sum() == 2 * c * c
