"""GPU: the entry point that allocates nothing (usp_attn_fwd_noalloc, scratch in a static device array) against
usp_attn_fwd with a caller workspace, through the C ABI: two calls in a row, the second with a smaller input; then
the size limit.  Same kernels on the same data: the outputs must agree bit for bit (and both match the oracle)."""
import numpy as np
import pytest
import torch

from oracle import usp_oracle as orc
from tests import usp_testlib as tl

pytestmark = pytest.mark.gpu


def _run_both(usp, seed, bs, L, hc, hk, hs, U, R):
    prob = tl.Problem(seed, bs, L, hc, hk, hs, U, R, True, True, tl.BF16)
    p = usp.problem(bs, L, hc, hk, hs, U, R, True, usp.USP_SPLIT_ZIGZAG, usp.USP_BF16)
    q, k, v = (prob.seq_layout_dev(n) for n in ("q", "k", "v"))
    outs = []
    for noalloc in (False, True):
        o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((prob.N, bs, hc // U, L // R), float("nan"), dtype=torch.float32, device="cuda")
        if noalloc:
            usp.usp_attn_fwd_noalloc(p, q, k, v, o, lse, 0, prob.N)
        else:
            ws = torch.empty(usp.usp_attn_fwd_workspace_bytes(p, prob.N), dtype=torch.uint8, device="cuda")
            usp.usp_attn_fwd(p, q, k, v, o, lse, 0, prob.N, ws)
        torch.cuda.synchronize()
        outs.append((o, lse))
    (o0, l0), (o1, l1) = outs
    assert torch.equal(o0.view(torch.int16), o1.view(torch.int16))
    assert torch.equal(l0.view(torch.int32), l1.view(torch.int32))
    ref_o, ref_l = orc.usp_attention_reference_by_rank(prob.val["q"], prob.val["k"], prob.val["v"], True, R, U, True)
    og, lg = tl.to_f64(o1), tl.to_f64(l1)
    for rank in range(prob.N):
        assert tl.max_abs(og[rank], ref_o[rank]) <= 2e-2
        tl.assert_lse_close(lg[rank], ref_l[rank], 1e-3)


def test_noalloc_forward_matches_workspace_forward_twice_then_smaller(usp):
    # a ring of 4 x Ulysses 2 (K/V staging of every block in the scratch), then a smaller problem of another shape
    # (short sequence: key-split path, fp32 partials in the scratch) over what the first call left there
    _run_both(usp, 71, 1, 4096, 8, 4, 128, 2, 4)
    _run_both(usp, 72, 2, 1024, 4, 2, 64, 2, 1)
    _run_both(usp, 73, 1, 2048, 8, 2, 128, 1, 2)


def test_noalloc_forward_rejects_problems_beyond_the_static_array(usp):
    p = usp.problem(1, 212992, 32, 8, 128, 8, 2, True)
    assert usp.usp_attn_fwd_workspace_bytes(p, 1) <= usp.USP_NOALLOC_SCRATCH_BYTES < usp.usp_attn_fwd_workspace_bytes(p, 16)
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(usp.UspError) as e:
        usp.usp_attn_fwd_noalloc(p, x, x, x, x, x, 0, 16)      # validated on the host: nothing is enqueued
    assert e.value.status == 5
    with pytest.raises(usp.UspError):
        usp.usp_attn_fwd_noalloc(p, x, x, x, x, x, 3, 3)       # empty rank range


def test_noalloc_forward_without_room_for_optional_partials(usp):
    """A rank whose heaviest query tiles usp_attn_fwd cuts into one item per ring block (four fp32 partial results, 240
    MiB of workspace in all): the entry point without a workspace has no room for those, leaves the launch whole and
    still gives the same attention (both against the oracle on sampled rows; the two differ only by rounding order)."""
    import tests.test_gpu_full_configs as full
    case = tl.OneRankCase(usp, 1234, 1, 98304, 32, 8, 128, 8, 4, 0)
    assert usp.usp_attn_fwd_workspace_bytes(case.p, 1) > usp.USP_NOALLOC_SCRATCH_BYTES
    case.forward()
    rows = case.sample_rows(np.random.default_rng(9), 96)
    full._check_forward_rows(case, rows)
    o_ws, lse_ws = case.o, case.lse
    case.o = torch.zeros_like(case.q)
    case.lse = torch.zeros_like(lse_ws)
    usp.usp_attn_fwd_noalloc(case.p, case.q, case.k, case.v, case.o, case.lse, case.rank, case.rank + 1)
    torch.cuda.synchronize()
    full._check_forward_rows(case, rows)
    assert float((case.o.float() - o_ws.float()).abs().max()) <= 2e-2
    assert float((case.lse[case.rank] - lse_ws[case.rank]).abs().max()) <= 1e-3

