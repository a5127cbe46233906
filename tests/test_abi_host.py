"""CPU-side checks of the C ABI: the library loads, exports what include/usp.h declares, and its
host-only entry points (validation, Algorithm 2 positions, workspace sizes) agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import usp_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def usp():
    import paper_2405_07719_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2405_07719_amd import build
        build.build(verbose=False)
    pkg.load()
    return pkg


def test_library_exports_every_declared_symbol(usp):
    header = open(os.path.join(ROOT, "include", "usp.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(usp_[a-z0-9_]+)\s*\(", header))
    assert {"usp_layout_a2a", "usp_block_attn_fwd", "usp_lse_merge", "usp_attn_fwd", "usp_attn_bwd",
            "usp_validate", "usp_local_positions", "usp_status_str"} <= names
    lib = ctypes.CDLL(usp.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in usp.h but not exported by libusp.so"


def test_struct_layouts_match_the_header(usp):
    # int32, (pad), int64, 8 x int32, float, (pad) -> 56 bytes; four int64 -> 32 bytes
    assert ctypes.sizeof(usp.usp_problem) == 56
    assert usp.usp_problem.L.offset == 8 and usp.usp_problem.scale.offset == 48
    assert ctypes.sizeof(usp.usp_posdesc) == 32


def test_validate_follows_the_paper_constraints(usp):
    ok = usp.problem(1, 32768, 32, 8, 128, 8, 1, True)
    assert usp.usp_validate(ok) == 0
    assert usp.usp_validate(usp.problem(1, 212992, 32, 8, 128, 8, 2, True)) == 0      # llama3-8B, SP 16 = 8 x 2
    assert usp.usp_validate(usp.problem(1, 32768, 32, 8, 128, 16, 1, True)) == 3      # U beyond the KV heads
    assert usp.usp_validate(usp.problem(1, 32768, 32, 1, 128, 2, 4, True)) == 3       # MQA: Ulysses cannot split
    assert usp.usp_validate(usp.problem(1, 32768, 32, 1, 128, 1, 8, True)) == 0       # ... but ring-only works
    assert usp.usp_validate(usp.problem(1, 32768, 32, 5, 128, 1, 1, True)) == 3       # hc % hk
    assert usp.usp_validate(usp.problem(1, 1004, 4, 4, 64, 2, 2, True)) == 2          # L % 2RU for zigzag
    assert usp.usp_validate(usp.problem(1, 1004, 4, 4, 64, 2, 2, True, usp.USP_SPLIT_CONTIG)) == 0
    assert usp.usp_validate(usp.problem(1, 1024, 4, 4, 96, 2, 2, True)) == 6          # head size
    assert usp.usp_validate(usp.problem(0, 1024, 4, 4, 64, 2, 2, True)) == 2
    assert usp.usp_validate(usp.problem(1, 1024, 4, 4, 64, 2, 2, True, dtype=7)) == 4
    assert "degree" in usp.usp_status_str(3)


@pytest.mark.parametrize("L,R,U,zz", [(16, 4, 1, True), (64, 2, 4, True), (96, 3, 2, True), (64, 1, 8, True),
                                      (64, 8, 1, True), (60, 3, 5, False), (64, 4, 2, False)])
def test_local_positions_match_algorithm2_oracle(usp, L, R, U, zz):
    p = usp.problem(1, L, 8 * U, 8 * U, 64, U, R, True, usp.USP_SPLIT_ZIGZAG if zz else usp.USP_SPLIT_CONTIG)
    for r in range(R):
        for u in range(U):
            shard, blk = usp.usp_local_positions(p, r, u)
            assert shard.positions() == orc.zigzag_positions(L, R, U, r, u, zz).tolist()
            assert blk.positions() == orc.ring_block_positions(L, R, r, zz).tolist()
    with pytest.raises(usp.UspError):
        usp.usp_local_positions(p, R, 0)


def test_workspace_query_is_host_only_and_scales_with_the_problem(usp):
    p = usp.problem(1, 32768, 32, 8, 128, 8, 1, True)
    one = usp.usp_attn_fwd_workspace_bytes(p, 1)
    # one K and one V block in head layout (8 MiB each); Q and O are read from / written to the shards directly
    assert one == 2 * 8 * 2**20
    assert usp.usp_attn_fwd_workspace_bytes(p, 8) > one
    ring = usp.problem(1, 32768, 32, 8, 128, 1, 8, True)
    w = usp.usp_attn_fwd_workspace_bytes(ring, 1)
    # bf16, R <= 16: the ring loop is one launch, and with Ulysses degree 1 the all-to-alls are the identity: a K/V block
    # in head layout is its shard as it stands, nothing is staged, no workspace at all
    assert w == 0
    # ... with Ulysses 2 x ring 4 the 4 K and 4 V blocks of a column are staged (16384 keys x 4 heads: 16 MiB each)
    assert usp.usp_attn_fwd_workspace_bytes(usp.problem(1, 65536, 32, 8, 128, 2, 4, True), 1) == 2 * 4 * 16 * 2**20
    # fp32 data runs one launch per ring step: Q and O in head layout (64 MiB each, elements are 4 bytes now; K/V in place),
    # 8 fp32 partial O and 8 partial LSE
    ring32 = usp.problem(1, 32768, 32, 8, 128, 1, 8, True, usp.USP_SPLIT_ZIGZAG, usp.USP_FP32)
    w32 = usp.usp_attn_fwd_workspace_bytes(ring32, 1)
    assert w32 == 2 * 64 * 2**20 + 8 * 64 * 2**20 + 8 * 2**19
    # more ring ranks than one launch takes blocks: partials again
    long_ring = usp.problem(1, 32768, 32, 8, 128, 1, 32, True)
    assert usp.usp_attn_fwd_workspace_bytes(long_ring, 1) == 2 * 8 * 2**20 + 32 * 16 * 2**20 + 32 * 2**17
    # a short sequence (128 work items for 256 CUs): each block is cut into 3 pieces that run side by side,
    # + 3 fp32 partial O (16 MiB each) and 3 partial LSE (128 KiB each)
    short = usp.problem(1, 8192, 32, 8, 128, 8, 1, True)
    assert usp.usp_attn_fwd_workspace_bytes(short, 1) == 2 * 2 * 2**20 + 3 * 16 * 2**20 + 3 * 2**17
    assert usp.usp_attn_fwd_workspace_bytes(p, 0) == 0
    # medium length (320 work items for 256 CUs, the heaviest longer than a CU's share): the last query tiles are cut in
    # two, which takes K and V as rows (5 MiB each) + 2 fp32 partial O (40 MiB each) + 2 partial LSE (320 KiB each) ...
    medium = usp.problem(1, 20480, 32, 8, 128, 8, 1, True)
    assert usp.usp_attn_fwd_workspace_bytes(medium, 1) == 2 * 5 * 2**20 + 2 * 40 * 2**20 + 2 * 320 * 2**10
    # ... longer still (448 items) a few tiles in three pieces (K rows and transposed V tiles of 7 MiB, 3 partials of
    # 56 MiB + 448 KiB), and from two items per CU on nothing (K and V, 8 MiB each)
    assert (usp.usp_attn_fwd_workspace_bytes(usp.problem(1, 28672, 32, 8, 128, 8, 1, True), 1)
            == 2 * 7 * 2**20 + 3 * (56 * 2**20 + 448 * 2**10))
    assert usp.usp_attn_fwd_workspace_bytes(usp.problem(1, 32768, 32, 8, 128, 8, 1, True), 1) == 2 * 8 * 2**20
    # without the causal mask the 320 items weigh the same and the second, quarter-filled round is what is lost:
    # some tiles in three pieces fill the first round instead (three partials)
    assert (usp.usp_attn_fwd_workspace_bytes(usp.problem(1, 20480, 32, 8, 128, 8, 1, False), 1)
            == 2 * 5 * 2**20 + 3 * 40 * 2**20 + 3 * 320 * 2**10)
    # backward: Q and dO in head layout (32 MiB each; O is only read for delta, straight from the shards), delta (0.5),
    # K and V (8 each), fp32 dQ (64) and one fp32 copy of dK and of dV (16 MiB each) per query head of the group: the
    # four heads run as separate work items
    assert usp.usp_attn_bwd_workspace_bytes(p, 1) == (2 * 32 + 2 * 8 + 64 + 2 * 4 * 16) * 2**20 + 2**19
    # the short sequence: 4 slices of the dQ items (4 copies of 16 MiB), 4 head splits x 4 query slices of dK/dV
    # (16 copies of 4 MiB each)
    assert usp.usp_attn_bwd_workspace_bytes(short, 1) == (2 * 8 + 2 * 2 + 4 * 16 + 2 * 16 * 4) * 2**20 + 2**17
    # with room for dS (bf16, one 32 x 32 block per 2 KiB, both lengths rounded up to 256): 4 heads x 32768^2 x 2 bytes more
    assert usp.usp_attn_bwd_workspace_bytes_with_ds(p, 1) - usp.usp_attn_bwd_workspace_bytes(p, 1) == 4 * 32768**2 * 2
    assert usp.usp_attn_bwd_workspace_bytes_with_ds(short, 1) - usp.usp_attn_bwd_workspace_bytes(short, 1) == 4 * 8192**2 * 2
    # the ring-only rank needs no head-layout copies at all: delta (0.5 MiB), fp32 dQ (64 MiB), and for each of the 8
    # blocks fp32 dK and dV (4096 keys x 8 heads: 16 MiB) in two copies
    assert usp.usp_attn_bwd_workspace_bytes(ring, 1) == 2**19 + (64 + 8 * 2 * 2 * 16) * 2**20
    # one rank of the ring: 32 heads, 8 blocks of 4096 keys for its 4096 queries
    assert (usp.usp_attn_bwd_workspace_bytes_with_ds(ring, 1) - usp.usp_attn_bwd_workspace_bytes(ring, 1)
            == 32 * 8 * 4096**2 * 2)
    # the per-call form: lengths that are no multiple of 256 are rounded up (333 -> 512 queries, 700 -> 768 keys)
    plain = usp.usp_ring_attn_bwd_workspace_bytes(2, 333, 700, 4, 2, 128, 3)
    assert usp.usp_ring_attn_bwd_workspace_bytes_with_ds(2, 333, 700, 4, 2, 128, 3) - plain == 2 * 4 * 3 * 512 * 768 * 2
    assert usp.usp_ring_attn_bwd_workspace_bytes_with_ds(2, 333, 700, 4, 3, 128, 3) == 0     # heads do not divide
    # head size 64: forming S and dP a second time is cheaper than moving dS, no room is asked for
    p64 = usp.problem(1, 32768, 32, 8, 64, 8, 1, True)
    assert usp.usp_attn_bwd_workspace_bytes_with_ds(p64, 1) == usp.usp_attn_bwd_workspace_bytes(p64, 1) > 0
    assert (usp.usp_ring_attn_bwd_workspace_bytes_with_ds(2, 333, 700, 4, 2, 64, 3)
            == usp.usp_ring_attn_bwd_workspace_bytes(2, 333, 700, 4, 2, 64, 3))


def test_loading_the_binding_first_leaves_one_hip_runtime_in_the_process():
    """torch ships a HIP runtime of its own; a process that loaded the library before torch once held two of them
    (the system's and torch's), and launches on torch's buffers then failed.  load() imports torch first."""
    import subprocess
    import sys
    code = ("import paper_2405_07719_amd as u; u.load(); import torch\n"
            "m = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}\n"
            "print(len(m))")
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    assert out.returncode == 0, out.stderr[-500:]
    assert out.stdout.strip() == "1"


def test_planning_a_known_problem_again_costs_the_host_next_to_nothing(usp):
    """usp_attn_fwd plans at every call; for medium lengths that includes playing the launch through on the host
    (a fraction of a millisecond), which is done once per problem and kept: repeated calls must not pay it again."""
    import time
    problems = [usp.problem(1, L, 32, 8, 128, 8, 1, True) for L in (20480, 24576, 32768)] + [usp.problem(1, 32768, 32, 8, 128, 1, 8, True)]
    for p in problems:
        usp.usp_attn_fwd_workspace_bytes(p, 1)
    t0 = time.perf_counter()
    for _ in range(200):
        for p in problems:
            usp.usp_attn_fwd_workspace_bytes(p, 1)
    assert (time.perf_counter() - t0) / 800 < 50e-6
