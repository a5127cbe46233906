"""CPU oracle for the USP attention path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy code that states what the GPU path must compute.  It is
imported only by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg; the product (the HIP library and its Python binding) never
imports it, and it imports nothing from the product.

What each function follows in the paper (arxiv 2405.07719):

* attention / attention_rows / block_attention -- Sec. 2, Eq. 1: softmax(Q K^T * scale) V
  per head, written out row by row over the *global* un-split tensors.  The causal
  mask is by global position; a GQA query head h reads KV head h // (hc // hk)
  (Sec. 3, the GQA/MQA paragraph).  LSE is the natural log of the softmax
  denominator (the paper never defines it; this is the usual definition).
* attention_backward -- the textbook gradient of Eq. 1 (the paper gives none).
* attention_backward_columns -- the same gradient for selected key columns only, from
  rows whose log-sum-exp and delta are given (for problems too large for the above).
* zigzag_positions -- Sec. 3, Algorithm 2: split the sequence into 2R chunks, ring
  rank r keeps chunks r and 2R-1-r, Ulysses rank u keeps the u-th of U equal pieces.
* a2a_seq_to_head / a2a_head_to_seq -- Sec. 3, Algorithm 1 steps 2-4 and 6
  (AllToAll4D inside one Ulysses group): merge L, partition hc, and back.
* lse_merge -- the combination rule implied by "distributed FlashAttention"
  (Sec. 2): partial results over disjoint key sets combine by log-sum-exp weights.
* usp_attention_reference_by_rank -- Algorithm 1 end to end, expressed through
  the definitions above (global attention, then pick each rank's rows): the
  distributed method reaches exactly this result.

Pins (tests/test_oracle_pins.py): brute-force loops on tiny inputs, closed forms
(Q = 0, constant V, single key), softmax normalisation, an independent library
routine on the un-masked/causal special cases, central finite differences for
the backward (also with scrambled explicit positions: scalar-loop gradient, central
differences of block_attention, a rank's rows = its share of the full gradient),
the paper's worked zigzag example (Sec. 3: 16 tokens, 4 GPUs, GPU0
holds tokens 0,1,14,15), the balanced pair count, the 7x imbalance of the even
split on 4 GPUs, and reshape/transpose second opinions for the layout maps.
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------- #
# Eq. 1: attention by global positions
# --------------------------------------------------------------------------- #
def _visible(qpos: np.ndarray, kpos: np.ndarray, causal: bool) -> np.ndarray:
    """Boolean [nq, nk]: key j is visible to query i (causal: kpos[j] <= qpos[i])."""
    if not causal:
        return np.ones((qpos.size, kpos.size), dtype=bool)
    return kpos[None, :] <= qpos[:, None]


def _attend_one_head(q, k, v, vis, scale):
    """One head.  q [nq, hs], k,v [nk, hs], vis bool [nq, nk] -> o [nq, hs], lse [nq].

    Rows with no visible key return o = 0 and lse = -inf.
    """
    s = (q @ k.T) * scale
    s = np.where(vis, s, NEG_INF)
    m = s.max(axis=1) if s.shape[1] else np.full(s.shape[0], NEG_INF)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m_safe[:, None])            # exp(-inf) = 0 for hidden keys
    denom = e.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        p = np.where(denom[:, None] > 0, e / denom[:, None], 0.0)
        lse = np.where(denom > 0, m_safe + np.log(denom), NEG_INF)
    return p @ v, lse


def block_attention(q, k, v, qpos, kpos, causal, scale=None, row_chunk=2048):
    """Attention of query rows against a set of keys, masked by global position.

    q [bs, nq, hq, hs]; k, v [bs, nk, hkv, hs]; qpos [nq], kpos [nk] global positions.
    Query head h uses KV head h // (hq // hkv).  Returns o [bs, nq, hq, hs] and
    lse [bs, hq, nq] (fp64).  Eq. 1 restricted to the given key set.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    qpos = np.asarray(qpos, dtype=np.int64)
    kpos = np.asarray(kpos, dtype=np.int64)
    bs, nq, hq, hs = q.shape
    hkv = k.shape[2]
    assert hq % hkv == 0 and k.shape == v.shape and k.shape[0] == bs and k.shape[3] == hs
    g = hq // hkv
    if scale is None:
        scale = 1.0 / math.sqrt(hs)
    o = np.zeros((bs, nq, hq, hs), dtype=np.float64)
    lse = np.full((bs, hq, nq), NEG_INF, dtype=np.float64)
    for b in range(bs):
        for h in range(hq):
            kh, vh = k[b, :, h // g, :], v[b, :, h // g, :]
            for r0 in range(0, nq, row_chunk):     # row chunks bound memory only; each row sees all keys at once
                r1 = min(nq, r0 + row_chunk)
                vis = _visible(qpos[r0:r1], kpos, causal)
                o[b, r0:r1, h, :], lse[b, h, r0:r1] = _attend_one_head(q[b, r0:r1, h, :], kh, vh, vis, scale)
    return o, lse


def attention(q, k, v, causal, scale=None):
    """Eq. 1 on global tensors: q [bs, L, hc, hs], k,v [bs, L, hk, hs] -> o, lse[bs, hc, L]."""
    L = q.shape[1]
    pos = np.arange(L, dtype=np.int64)
    return block_attention(q, k, v, pos, np.arange(k.shape[1], dtype=np.int64), causal, scale)


def attention_rows(q_rows, row_pos, k, v, causal, scale=None):
    """Eq. 1 for selected query rows only: q_rows [bs, n, hc, hs] at global positions row_pos."""
    return block_attention(q_rows, k, v, row_pos, np.arange(k.shape[1], dtype=np.int64), causal, scale)


# --------------------------------------------------------------------------- #
# Backward of Eq. 1 (textbook)
# --------------------------------------------------------------------------- #
def attention_backward(q, k, v, d_o, causal, scale=None, qpos=None, kpos=None):
    """Gradients of sum(O * dO) w.r.t. q, k, v for Eq. 1 (masked by position).

    With P = softmax(S), S = scale * Q K^T:  dV = P^T dO;  dP = dO V^T;
    dS = P * (dP - rowsum(dP * P));  dQ = scale * dS K;  dK = scale * dS^T Q.
    dK, dV of a KV head sum over the query heads of its group.
    Returns dq [bs,nq,hq,hs], dk, dv [bs,nk,hkv,hs].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    bs, nq, hq, hs = q.shape
    nk, hkv = k.shape[1], k.shape[2]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / math.sqrt(hs)
    qpos = np.arange(nq, dtype=np.int64) if qpos is None else np.asarray(qpos, dtype=np.int64)
    kpos = np.arange(nk, dtype=np.int64) if kpos is None else np.asarray(kpos, dtype=np.int64)
    vis = _visible(qpos, kpos, causal)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(bs):
        for h in range(hq):
            kh, vh = k[b, :, h // g, :], v[b, :, h // g, :]
            qh, doh = q[b, :, h, :], d_o[b, :, h, :]
            s = np.where(vis, (qh @ kh.T) * scale, NEG_INF)
            m = s.max(axis=1)
            m_safe = np.where(np.isfinite(m), m, 0.0)
            e = np.exp(s - m_safe[:, None])
            den = e.sum(axis=1)
            with np.errstate(divide="ignore", invalid="ignore"):
                p = np.where(den[:, None] > 0, e / den[:, None], 0.0)
            dp = doh @ vh.T
            ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            dq[b, :, h, :] = scale * (ds @ kh)
            dk[b, :, h // g, :] += scale * (ds.T @ qh)
            dv[b, :, h // g, :] += p.T @ doh
    return dq, dk, dv


def attention_backward_columns(q, d_o, lse, delta, qpos, k_cols, v_cols, col_pos, causal, scale=None):
    """dK, dV of SELECTED key columns from the given query rows (textbook gradient of Eq. 1, column by column).

    For problems too large for attention_backward: the softmax of a row is fixed by its log-sum-exp over ALL its
    visible keys, so with lse [bs, hq, nq] (from block_attention over every key) and delta_i = sum_e dO_ie O_ie
    [bs, hq, nq] the weight of one (row, key) pair needs nothing else:
      P_ij = exp(scale q_i.k_j - lse_i) if key j is visible to row i, else 0
      dV_j = sum_i P_ij dO_i;   dS_ij = P_ij (dO_i.v_j - delta_i);   dK_j = scale sum_i dS_ij q_i
    summed over the query heads of the KV head's group.  q, d_o [bs, nq, hq, hs] at positions qpos; k_cols, v_cols
    [bs, nc, hkv, hs] at positions col_pos.  Returns dk, dv [bs, nc, hkv, hs]: the given rows' contribution.
    """
    q = np.asarray(q, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    k_cols = np.asarray(k_cols, dtype=np.float64)
    v_cols = np.asarray(v_cols, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64)
    delta = np.asarray(delta, dtype=np.float64)
    bs, nq, hq, hs = q.shape
    hkv = k_cols.shape[2]
    g = hq // hkv
    if scale is None:
        scale = 1.0 / math.sqrt(hs)
    vis = _visible(np.asarray(qpos, dtype=np.int64), np.asarray(col_pos, dtype=np.int64), causal)
    dk = np.zeros_like(k_cols)
    dv = np.zeros_like(v_cols)
    for b in range(bs):
        for h in range(hq):
            kh, vh = k_cols[b, :, h // g, :], v_cols[b, :, h // g, :]
            qh, doh = q[b, :, h, :], d_o[b, :, h, :]
            live = np.isfinite(lse[b, h])                               # rows that see no key at all have P = 0
            with np.errstate(invalid="ignore"):
                p = np.where(vis & live[:, None], np.exp((qh @ kh.T) * scale - np.where(live, lse[b, h], 0.0)[:, None]), 0.0)
            ds = p * (doh @ vh.T - delta[b, h][:, None])
            dk[b, :, h // g, :] += scale * (ds.T @ qh)
            dv[b, :, h // g, :] += p.T @ doh
    return dk, dv


# --------------------------------------------------------------------------- #
# Algorithm 2: which global positions a virtual rank holds
# --------------------------------------------------------------------------- #
def ring_block_positions(L, ring, r, zigzag=True):
    """Global positions of ring rank r's sequence block (length L // ring), in local order.

    zigzag: concat(chunk[r], chunk[2R-1-r]) with 2R chunks (Algorithm 2);
    otherwise the contiguous block r of R (the "basic ring" split).
    """
    if zigzag:
        assert L % (2 * ring) == 0
        c = L // (2 * ring)
        return np.concatenate([np.arange(r * c, (r + 1) * c), np.arange((2 * ring - 1 - r) * c, (2 * ring - r) * c)]).astype(np.int64)
    assert L % ring == 0
    n = L // ring
    return np.arange(r * n, (r + 1) * n, dtype=np.int64)


def zigzag_positions(L, ring, ulysses, r, u, zigzag=True):
    """Global positions of the input shard of virtual rank (r, u): the u-th of U equal pieces of ring block r."""
    blk = ring_block_positions(L, ring, r, zigzag)
    assert blk.size % ulysses == 0
    n = blk.size // ulysses
    return blk[u * n:(u + 1) * n]


def causal_pair_count(qpos, kpos):
    """Number of (query, key) pairs with kpos <= qpos (the work a causal kernel must do)."""
    kp = np.sort(np.asarray(kpos, dtype=np.int64))
    return int(np.searchsorted(kp, np.asarray(qpos, dtype=np.int64), side="right").sum())


# --------------------------------------------------------------------------- #
# Algorithm 1 steps 2-4 / 6: the Ulysses all-to-all as an index map
# --------------------------------------------------------------------------- #
def a2a_seq_to_head(shards, u):
    """shards: list over u' of [bs, n, h, hs] (the Ulysses group's seq-layout shards, ascending rank).

    Returns rank u's head-layout tensor Y [bs, U*n, h/U, hs] with
    Y[b, u'*n + s, h', e] = shards[u'][b, s, u*(h/U) + h', e].
    """
    U = len(shards)
    bs, n, h, hs = shards[0].shape
    assert h % U == 0
    hl = h // U
    y = np.empty((bs, U * n, hl, hs), dtype=shards[0].dtype)
    for up in range(U):
        for s in range(n):
            for hp in range(hl):
                y[:, up * n + s, hp, :] = shards[up][:, s, u * hl + hp, :]
    return y


def a2a_head_to_seq(heads):
    """heads: list over u of [bs, U*n, h/U, hs] (head-layout tensors of one Ulysses group).

    Returns the list over u' of seq-layout shards X_{u'} [bs, n, h, hs] with
    X_{u'}[b, s, u*(h/U) + h', e] = heads[u][b, u'*n + s, h', e]  (inverse of a2a_seq_to_head).
    """
    U = len(heads)
    bs, ln, hl, hs = heads[0].shape
    assert ln % U == 0
    n = ln // U
    out = [np.empty((bs, n, hl * U, hs), dtype=heads[0].dtype) for _ in range(U)]
    for up in range(U):
        for u in range(U):
            for s in range(n):
                for hp in range(hl):
                    out[up][:, s, u * hl + hp, :] = heads[u][:, up * n + s, hp, :]
    return out


# --------------------------------------------------------------------------- #
# Merge of partial results over disjoint key sets
# --------------------------------------------------------------------------- #
def lse_merge(o_parts, lse_parts):
    """o_parts: list of [bs, n, hq, hs]; lse_parts: list of [bs, hq, n] -> merged (o, lse).

    LSE = ln sum_i exp(LSE_i);  O = sum_i exp(LSE_i - LSE) O_i.  Parts with
    LSE_i = -inf contribute nothing; if all are -inf the row is (0, -inf).
    """
    o_parts = [np.asarray(o, dtype=np.float64) for o in o_parts]
    lse_parts = [np.asarray(l, dtype=np.float64) for l in lse_parts]
    stack = np.stack(lse_parts)                            # [n_parts, bs, hq, n]
    m = stack.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    tot = np.exp(stack - m_safe[None]).sum(axis=0)
    with np.errstate(divide="ignore"):
        lse = np.where(tot > 0, m_safe + np.log(tot), NEG_INF)
    o = np.zeros_like(o_parts[0])
    for op, lp in zip(o_parts, lse_parts):
        with np.errstate(invalid="ignore"):
            w = np.where(np.isfinite(lp), np.exp(lp - np.where(np.isfinite(lse), lse, 0.0)), 0.0)   # [bs, hq, n]
        o += np.transpose(w, (0, 2, 1))[..., None] * op
    return o, lse


# --------------------------------------------------------------------------- #
# Algorithm 1 end to end, through the definitions
# --------------------------------------------------------------------------- #
def usp_attention_reference_by_rank(q, k, v, causal, ring, ulysses, zigzag=True, scale=None):
    """What every virtual rank must end up holding after Algorithm 1.

    q [bs, L, hc, hs], k, v [bs, L, hk, hs] are the GLOBAL tensors.  Returns
    (o_shards, lse_heads): o_shards[rank] = O at the rank's Algorithm-2 positions,
    all heads, [bs, L/N, hc, hs]; lse_heads[rank] = LSE of the rank's local heads
    over its ring block, [bs, hc/U, L/R]; rank = r * U + u.
    """
    L, hc = q.shape[1], q.shape[2]
    o, lse = attention(q, k, v, causal, scale)
    hl = hc // ulysses
    o_shards, lse_heads = [], []
    for r in range(ring):
        blk = ring_block_positions(L, ring, r, zigzag)
        for u in range(ulysses):
            o_shards.append(o[:, zigzag_positions(L, ring, ulysses, r, u, zigzag), :, :])
            lse_heads.append(lse[:, u * hl:(u + 1) * hl, :][:, :, blk])
    return o_shards, lse_heads
