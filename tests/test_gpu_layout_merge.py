"""GPU parity: the Ulysses layout transform (bit-exact) and the LSE merge, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from tests import usp_testlib as tl

pytestmark = pytest.mark.gpu


def _tags(shape, dtype):
    """Distinct integer tags per element (as raw bits) so that any misplaced element is caught."""
    n = int(np.prod(shape))
    if dtype == tl.BF16:
        return (np.arange(n, dtype=np.uint64) * np.uint64(2654435761) % np.uint64(65521)).astype(np.uint16).reshape(shape)
    return np.arange(n, dtype=np.uint32).view(np.float32).reshape(shape)


def _bits(t):
    t = t.cpu()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy().view(np.uint32)


@pytest.mark.parametrize("bs,L,heads,hs,U,R,dtype", [
    (1, 256, 4, 64, 2, 2, tl.FP32),        # config-1 shape
    (2, 96, 8, 64, 4, 1, tl.BF16),
    (1, 4096, 32, 128, 8, 1, tl.BF16),     # Q of the Ulysses-only config, scaled down in L
    (1, 4096, 8, 128, 8, 1, tl.BF16),      # K/V of the same: one KV head per rank, 256 B runs
    (1, 1200, 6, 128, 3, 2, tl.BF16),      # non power-of-two runs, ragged against the block size
    (3, 64, 4, 128, 1, 4, tl.BF16),        # U = 1: identity
    (1, 2048, 16, 128, 2, 4, tl.BF16),     # training config shape, scaled down
])
def test_layout_a2a_bit_exact_and_round_trip(usp, bs, L, heads, hs, U, R, dtype):
    N = U * R
    p = usp.problem(bs, L, heads, heads, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, dtype)
    n = L // N
    seq = _tags((N, bs, n, heads, hs), dtype)
    src = tl.to_device(seq, dtype)
    head = torch.zeros((N, bs, L // R, heads // U, hs), dtype=src.dtype, device="cuda")
    usp.usp_layout_a2a(p, heads, usp.USP_SEQ_TO_HEAD, src, head, 0, N)
    torch.cuda.synchronize()
    got = _bits(head)
    seq_bits = _bits(src)
    for r in range(R):
        shards = [seq_bits[r * U + up] for up in range(U)]
        for u in range(U):
            assert np.array_equal(got[r * U + u], orc.a2a_seq_to_head(shards, u)), (r, u)
    if U == 1:
        assert np.array_equal(got, seq_bits.reshape(got.shape))
    back = torch.zeros_like(src)
    usp.usp_layout_a2a(p, heads, usp.USP_HEAD_TO_SEQ, head, back, 0, N)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(back), seq_bits)


def test_layout_a2a_rank_subrange_touches_only_its_ranks(usp):
    bs, L, heads, hs, U, R = 1, 512, 8, 64, 4, 2
    N = U * R
    p = usp.problem(bs, L, heads, heads, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, tl.BF16)
    seq = _tags((N, bs, L // N, heads, hs), tl.BF16)
    src = tl.to_device(seq, tl.BF16)
    head = torch.full((N, bs, L // R, heads // U, hs), -1.0, dtype=torch.bfloat16, device="cuda")
    usp.usp_layout_a2a(p, heads, usp.USP_SEQ_TO_HEAD, src, head, 5, 7)
    torch.cuda.synchronize()
    got = _bits(head)
    sentinel = _bits(torch.full((1,), -1.0, dtype=torch.bfloat16))[0]
    for rank in range(N):
        if rank in (5, 6):
            r, u = divmod(rank, U)
            assert np.array_equal(got[rank], orc.a2a_seq_to_head([seq[r * U + up] for up in range(U)], u))
        else:
            assert np.all(got[rank] == sentinel)
    # reverse direction from the same two ranks fills only their head slices of ring row 1's shards
    back = torch.full_like(src, -1.0)
    usp.usp_layout_a2a(p, heads, usp.USP_HEAD_TO_SEQ, head, back, 5, 7)
    torch.cuda.synchronize()
    bb = _bits(back)
    hl = heads // U
    for rank in range(N):
        for h in range(heads):
            owner = (rank // U) * U + h // hl
            if owner in (5, 6):
                assert np.array_equal(bb[rank][:, :, h], seq[rank][:, :, h])
            else:
                assert np.all(bb[rank][:, :, h] == sentinel)


def test_layout_a2a_rejects_bad_arguments(usp):
    p = usp.problem(1, 256, 8, 8, 64, 4, 2, True)
    x = torch.zeros(16, device="cuda")
    with pytest.raises(usp.UspError) as e:
        usp.usp_layout_a2a(p, 6, usp.USP_SEQ_TO_HEAD, x, x, 0, 8)       # heads % U != 0
    assert e.value.status == 3
    with pytest.raises(usp.UspError):
        usp.usp_layout_a2a(p, 8, usp.USP_SEQ_TO_HEAD, x, x, 0, 9)       # rank range beyond N
    with pytest.raises(usp.UspError):
        usp.usp_layout_a2a(p, 8, 7, x, x, 0, 8)                          # unknown direction
    with pytest.raises(usp.UspError):
        usp.usp_layout_a2a(p, 8, usp.USP_SEQ_TO_HEAD, None, x, 0, 8)    # null pointer


# ------------------------------------------------------------------------------------- merge
def _rand_parts(rng, n, bs, Lq, hq, hs, neg_inf_frac=0.0):
    o = [rng.standard_normal((bs, Lq, hq, hs)).astype(np.float32) for _ in range(n)]
    lse = [(rng.standard_normal((bs, hq, Lq)) * 3).astype(np.float32) for _ in range(n)]
    if neg_inf_frac:
        for i in range(n):
            dead = rng.random((bs, hq, Lq)) < neg_inf_frac
            lse[i][dead] = -np.inf
            o[i][np.transpose(dead, (0, 2, 1))] = 0.0
    return o, lse


@pytest.mark.parametrize("n,bs,Lq,hq,hs,out_dtype", [
    (2, 1, 128, 2, 64, tl.FP32),
    (8, 1, 1000, 4, 128, tl.BF16),      # ragged against the 256-thread workgroup
    (4, 2, 333, 3, 128, tl.FP32),
    (1, 1, 77, 5, 64, tl.FP32),
    (5, 1, 64, 32, 128, tl.BF16),       # more heads than positions
    (12, 1, 100, 2, 64, tl.FP32),       # more than eight parts: the general (looping) instance
    (3, 2, 50, 4, 128, tl.BF16),
])
def test_lse_merge_matches_oracle(usp, n, bs, Lq, hq, hs, out_dtype):
    rng = np.random.default_rng(11 + n)
    o, lse = _rand_parts(rng, n, bs, Lq, hq, hs, neg_inf_frac=0.2)
    # make a few rows dead in every part
    for i in range(n):
        lse[i][:, :, :3] = -np.inf
        o[i][:, :3] = 0.0
    ref_o, ref_l = orc.lse_merge(o, lse)
    d_o = [torch.from_numpy(x).cuda() for x in o]
    d_l = [torch.from_numpy(x).cuda() for x in lse]
    out = torch.empty((bs, Lq, hq, hs), dtype=torch.float32 if out_dtype == tl.FP32 else torch.bfloat16, device="cuda")
    out_l = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_lse_merge(d_o, d_l, out, out_l, bs, Lq, hq, hs, tl.FP32, out_dtype)
    torch.cuda.synchronize()
    tl.assert_lse_close(tl.to_f64(out_l), ref_l, 1e-5)
    tol = 1e-5 if out_dtype == tl.FP32 else 2e-2
    assert tl.max_abs(tl.to_f64(out), ref_o) <= tol
    assert np.all(tl.to_f64(out)[:, :3] == 0.0)


def test_lse_merge_bf16_parts_and_nan_payload_in_dead_part(usp):
    rng = np.random.default_rng(5)
    n, bs, Lq, hq, hs = 3, 1, 200, 2, 64
    o, lse = _rand_parts(rng, n, bs, Lq, hq, hs)
    from paper_2405_07719_amd import inputs
    ob = [inputs.to_bf16_bits(x) for x in o]
    ov = [inputs.from_bf16_bits(x) for x in ob]
    lse[1][:] = -np.inf                                   # a step that saw nothing ...
    ov[1][:] = 0.0
    ref_o, ref_l = orc.lse_merge(ov, lse)
    d_o = [tl.to_device(x, tl.BF16) for x in ob]
    d_o[1].fill_(float("nan"))                            # ... may hold anything: it must be erased, not multiplied
    d_l = [torch.from_numpy(x).cuda() for x in lse]
    out = torch.empty((bs, Lq, hq, hs), dtype=torch.float32, device="cuda")
    out_l = torch.empty((bs, hq, Lq), dtype=torch.float32, device="cuda")
    usp.usp_lse_merge(d_o, d_l, out, out_l, bs, Lq, hq, hs, tl.BF16, tl.FP32)
    torch.cuda.synchronize()
    tl.assert_lse_close(tl.to_f64(out_l), ref_l, 1e-5)
    assert tl.max_abs(tl.to_f64(out), ref_o) <= 1e-5


def test_lse_merge_rejects_bad_arguments(usp):
    x = torch.zeros(64, device="cuda")
    with pytest.raises(usp.UspError):
        usp.usp_lse_merge([], [], x, x, 1, 1, 1, 64, tl.FP32, tl.FP32)
    with pytest.raises(usp.UspError):
        usp.usp_lse_merge([x] * 65, [x] * 65, x, x, 1, 1, 1, 64, tl.FP32, tl.FP32)
    with pytest.raises(usp.UspError):
        usp.usp_lse_merge([x], [x], x, x, 1, 1, 1, 64, 9, tl.FP32)


# ------------------------------------------------------------------------------------- layout at the sizes bench.py times
def _big_tags(shape, mult):
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 26
    for a in range(0, n, step):                          # in pieces: the 64-bit intermediates of 872 M elements are 7 GB
        i = np.arange(a, min(n, a + step), dtype=np.uint64)
        out[a:a + i.size] = (i * np.uint64(mult) % np.uint64(65521)).astype(np.uint16)
    return out.reshape(shape)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,L,U,R,heads", [
    ("config2_q_all_8_ranks", 32768, 8, 1, 32),
    ("config4_q_all_16_ranks", 212992, 8, 2, 32),
    ("config4_k_all_16_ranks", 212992, 8, 2, 8),
])
def test_layout_a2a_bit_exact_at_bench_sizes(usp, name, L, U, R, heads):
    """The all-ranks launches bench.py times (512 MiB of traffic at config 2, 3.3 GiB at config 4), both directions,
    bit-exact against the oracle's index map on ranks 0, N/2 and N-1 and on their Ulysses groups."""
    bs, hs, N = 1, 128, U * R
    p = usp.problem(bs, L, heads, heads, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, tl.BF16)
    n, hl = L // N, heads // U
    seq = _big_tags((N, bs, n, heads, hs), 2654435761)
    src = tl.to_device(seq, tl.BF16)
    head = torch.zeros((N, bs, L // R, hl, hs), dtype=torch.bfloat16, device="cuda")
    usp.usp_layout_a2a(p, heads, usp.USP_SEQ_TO_HEAD, src, head, 0, N)
    torch.cuda.synchronize()
    for rank in (0, N // 2, N - 1):
        r, u = divmod(rank, U)
        ref = orc.a2a_seq_to_head([seq[r * U + up] for up in range(U)], u)
        assert np.array_equal(_bits(head[rank]), ref), rank
    del src
    # the reverse direction from head-layout tags of its own
    htags = _big_tags((N, bs, L // R, hl, hs), 40503)
    hsrc = tl.to_device(htags, tl.BF16)
    back = torch.zeros((N, bs, n, heads, hs), dtype=torch.bfloat16, device="cuda")
    usp.usp_layout_a2a(p, heads, usp.USP_HEAD_TO_SEQ, hsrc, back, 0, N)
    torch.cuda.synchronize()
    for r in sorted({0, R - 1}):
        ref = orc.a2a_head_to_seq([htags[r * U + u] for u in range(U)])
        for up in range(U):
            assert np.array_equal(_bits(back[r * U + up]), ref[up]), (r, up)


def test_lse_merge_in_place_on_part_0_and_rejected_overlaps(usp):
    """Outputs aliasing part 0: allowed (and correct) with equal dtypes at head size 64 / 128; rejected when the
    element sizes differ, at other head sizes, or when the buffers overlap without being the same."""
    rng = np.random.default_rng(9)
    for hs in (128, 64):
        n, bs, Lq, hq = 3, 2, 333, 3
        o, lse = _rand_parts(rng, n, bs, Lq, hq, hs, neg_inf_frac=0.1)
        ref_o, ref_l = orc.lse_merge(o, lse)
        d_o = [torch.from_numpy(x).cuda() for x in o]
        d_l = [torch.from_numpy(x).cuda() for x in lse]
        usp.usp_lse_merge(d_o, d_l, d_o[0], d_l[0], bs, Lq, hq, hs, tl.FP32, tl.FP32)       # in place on part 0
        torch.cuda.synchronize()
        tl.assert_lse_close(tl.to_f64(d_l[0]), ref_l, 1e-5)
        assert tl.max_abs(tl.to_f64(d_o[0]), ref_o) <= 1e-5
    x = torch.zeros((1, 64, 2, 128), dtype=torch.float32, device="cuda")
    l = torch.zeros((1, 2, 64), dtype=torch.float32, device="cuda")
    l2 = torch.zeros_like(l)
    with pytest.raises(usp.UspError) as e:            # fp32 part, bf16 output in the same buffer
        usp.usp_lse_merge([x], [l], x, l2, 1, 64, 2, 128, tl.FP32, tl.BF16)
    assert e.value.status == 6
    flat = torch.zeros(2 * x.numel(), dtype=torch.float32, device="cuda")
    with pytest.raises(usp.UspError):                 # overlapping, not identical
        usp.usp_lse_merge([flat[:x.numel()]], [l], flat[16:], l2, 1, 64, 2, 128, tl.FP32, tl.FP32)
    y = torch.zeros((1, 64, 2, 40), dtype=torch.float32, device="cuda")
    with pytest.raises(usp.UspError):                 # head size 40: a row's threads straddle wavefronts
        usp.usp_lse_merge([y], [l], y, l2, 1, 64, 2, 40, tl.FP32, tl.FP32)
    usp.usp_lse_merge([y], [l], torch.empty_like(y), l2, 1, 64, 2, 40, tl.FP32, tl.FP32)   # ... but fine out of place
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------- key-tile-transposed head layout
_VT_ORDER = np.array([0, 1, 2, 3, 8, 9, 10, 11, 4, 5, 6, 7, 12, 13, 14, 15])


def vt_of_head_layout(head):
    """The format of USP_SEQ_TO_HEAD_VT written out: head [bs, Lq, h, hs] -> [bs, h, tiles, hs, 64], place j of tile t
    = row 64 t + 16 (j // 16) + order[j % 16], zeros past the last row."""
    bs, Lq, h, hs = head.shape
    tiles = (Lq + 63) // 64
    padded = np.zeros((bs, tiles * 64, h, hs), dtype=head.dtype)
    padded[:, :Lq] = head
    j = np.arange(64)
    src = 16 * (j // 16) + _VT_ORDER[j % 16]
    t = padded.reshape(bs, tiles, 64, h, hs)[:, :, src]          # [bs, tiles, place, h, hs]
    return np.ascontiguousarray(np.transpose(t, (0, 3, 1, 4, 2)))  # [bs, h, tiles, hs, place]


@pytest.mark.parametrize("bs,L,heads,hs,U,R", [
    (1, 4096, 8, 128, 8, 1),      # K/V of the Ulysses-only config, scaled down
    (2, 1200, 6, 128, 3, 2),      # ring blocks of 600 rows: a ragged last tile (24 rows), shards of 200 rows
    (1, 2048, 16, 64, 2, 4),      # head size 64
    (3, 80, 4, 128, 1, 4),        # blocks shorter than one tile
])
def test_layout_a2a_transposed_tiles_bit_exact(usp, bs, L, heads, hs, U, R):
    N = U * R
    p = usp.problem(bs, L, heads, heads, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, tl.BF16)
    n, Lq, hl = L // N, L // R, heads // U
    seq = _tags((N, bs, n, heads, hs), tl.BF16)
    src = tl.to_device(seq, tl.BF16)
    tiles = (Lq + 63) // 64
    vt = torch.full((N, bs, hl, tiles, hs, 64), -1.0, dtype=torch.bfloat16, device="cuda")
    usp.usp_layout_a2a(p, heads, usp.USP_SEQ_TO_HEAD_VT, src, vt, 0, N)
    torch.cuda.synchronize()
    got = _bits(vt)
    for r in range(R):
        for u in range(U):
            head = orc.a2a_seq_to_head([seq[r * U + up] for up in range(U)], u)      # the oracle's all-to-all ...
            assert np.array_equal(got[r * U + u], vt_of_head_layout(head)), (r, u)    # ... in the tile format
    # a sub-range touches only its ranks
    vt2 = torch.full_like(vt, -1.0)
    usp.usp_layout_a2a(p, heads, usp.USP_SEQ_TO_HEAD_VT, src, vt2, N - 1, N)
    torch.cuda.synchronize()
    got2 = _bits(vt2)
    sentinel = _bits(torch.full((1,), -1.0, dtype=torch.bfloat16))[0]
    assert np.array_equal(got2[N - 1], got[N - 1]) and np.all(got2[:N - 1] == sentinel)
