"""USP (Ulysses x Ring) sequence-parallel attention hot path for MI355X (gfx950).

Thin ctypes binding over the C-ABI library `libusp.so` (declared in include/usp.h).
The functions here have the C names and do argument marshalling only: every step
of the path runs in the library's HIP kernels.  There is no CPU fallback: if the
library has not been built, `load()` (and therefore every call) raises.

Tensor arguments may be torch tensors (their `data_ptr()` is passed) or integers
holding device addresses; `stream` defaults to torch's current HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libusp.so")

USP_OK = 0
USP_BF16, USP_FP32 = 0, 1
USP_SPLIT_CONTIG, USP_SPLIT_ZIGZAG = 0, 1
USP_SEQ_TO_HEAD, USP_HEAD_TO_SEQ, USP_SEQ_TO_HEAD_VT = 0, 1, 2
USP_MAX_MERGE_PARTS = 64
USP_MAX_RING_BLOCKS = 16


class usp_problem(C.Structure):
    _fields_ = [("bs", C.c_int32), ("L", C.c_int64), ("hc", C.c_int32), ("hk", C.c_int32), ("hs", C.c_int32),
                ("ulysses", C.c_int32), ("ring", C.c_int32), ("causal", C.c_int32), ("split", C.c_int32),
                ("dtype", C.c_int32), ("scale", C.c_float)]


class usp_posdesc(C.Structure):
    _fields_ = [("start0", C.c_int64), ("len0", C.c_int64), ("start1", C.c_int64), ("len1", C.c_int64)]

    def positions(self):
        return list(range(self.start0, self.start0 + self.len0)) + list(range(self.start1, self.start1 + self.len1))


class UspError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: usp_status {status} ({usp_status_str(status)})")


_lib = None


def load():
    """Load libusp.so and declare its signatures.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2405_07719_amd.build` "
                           "(there is no CPU fallback)")
    # torch first: it ships a HIP runtime of its own, and the tensors and streams passed in belong to that one.
    # Loaded after torch, the library binds to the runtime already in the process; loaded before it, the library
    # would bring in the system's copy, torch its own, and launches on torch's buffers fail ("HIP launch error").
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    P, I, L, F, V = C.POINTER, C.c_int, C.c_int64, C.c_float, C.c_void_p
    lib.usp_status_str.restype = C.c_char_p
    lib.usp_status_str.argtypes = [I]
    lib.usp_validate.argtypes = [P(usp_problem)]
    lib.usp_local_positions.argtypes = [P(usp_problem), I, I, P(usp_posdesc), P(usp_posdesc)]
    lib.usp_layout_a2a.argtypes = [P(usp_problem), I, I, V, V, I, I, V]
    lib.usp_block_attn_fwd.argtypes = [V, V, V, V, V, I, L, L, I, I, I, F, I, P(usp_posdesc), P(usp_posdesc), I, I, V]
    lib.usp_block_attn_fwd_state_bytes.restype = C.c_size_t
    lib.usp_block_attn_fwd_state_bytes.argtypes = [I, L, I, I]
    lib.usp_block_attn_fwd_state.argtypes = [V, V, V, V, C.c_size_t, V, V, I, L, L, I, I, I, F, I, P(usp_posdesc),
                                             P(usp_posdesc), I, I, I, V]
    lib.usp_block_attn_fwd_state.restype = I
    lib.usp_lse_merge.argtypes = [P(V), P(V), I, V, V, I, L, I, I, I, I, V]
    lib.usp_ring_attn_fwd.argtypes = [V, P(V), P(V), P(usp_posdesc), I, V, V, I, L, L, I, I, I, F, I, P(usp_posdesc),
                                      I, I, V]
    lib.usp_ring_attn_fwd_vt.argtypes = [V, P(V), P(V), P(usp_posdesc), I, V, V, I, L, L, I, I, I, F, I, P(usp_posdesc), V]
    lib.usp_ring_attn_fwd_vt.restype = I
    lib.usp_ring_attn_fwd_partials.argtypes = [V, P(V), P(V), P(usp_posdesc), P(C.c_int32), I, P(V), P(V), I, L, L, I, I,
                                               I, F, I, P(usp_posdesc), V]
    lib.usp_attn_fwd_workspace_bytes.restype = C.c_size_t
    lib.usp_attn_fwd_workspace_bytes.argtypes = [P(usp_problem), I]
    lib.usp_attn_fwd.argtypes = [P(usp_problem), V, V, V, V, V, I, I, V, C.c_size_t, V]
    lib.usp_attn_fwd_noalloc.argtypes = [P(usp_problem), V, V, V, V, V, I, I, V]
    lib.usp_attn_fwd_noalloc.restype = I
    lib.usp_attn_delta.argtypes = [V, V, V, I, L, I, I, V]
    lib.usp_block_attn_bwd.argtypes = [V, V, V, V, V, V, V, V, V, I, L, L, I, I, I, F, I, P(usp_posdesc), P(usp_posdesc),
                                       I, V]
    lib.usp_ring_attn_bwd.argtypes = [V, P(V), P(V), P(usp_posdesc), I, V, V, V, V, P(V), P(V), I, L, L, I, I, I, F, I,
                                      P(usp_posdesc), I, P(I), V]
    lib.usp_ring_attn_bwd_workspace_bytes.restype = C.c_size_t
    lib.usp_ring_attn_bwd_workspace_bytes.argtypes = [I, L, L, I, I, I, I]
    lib.usp_ring_attn_bwd_workspace_bytes_with_ds.restype = C.c_size_t
    lib.usp_ring_attn_bwd_workspace_bytes_with_ds.argtypes = [I, L, L, I, I, I, I]
    lib.usp_ring_attn_bwd_ws.argtypes = [V, P(V), P(V), P(usp_posdesc), I, V, V, V, V, P(V), P(V), I, L, L, I, I, I, F, I,
                                         P(usp_posdesc), I, P(I), V, C.c_size_t, V]
    lib.usp_attn_bwd_workspace_bytes.restype = C.c_size_t
    lib.usp_attn_bwd_workspace_bytes.argtypes = [P(usp_problem), I]
    lib.usp_attn_bwd_workspace_bytes_with_ds.restype = C.c_size_t
    lib.usp_attn_bwd_workspace_bytes_with_ds.argtypes = [P(usp_problem), I]
    lib.usp_attn_bwd.argtypes = [P(usp_problem), V, V, V, V, V, V, V, V, V, I, I, V, C.c_size_t, V]
    for name in ("usp_ring_attn_bwd", "usp_ring_attn_fwd", "usp_validate", "usp_local_positions", "usp_layout_a2a", "usp_block_attn_fwd", "usp_lse_merge",
                 "usp_attn_fwd", "usp_attn_bwd", "usp_attn_delta", "usp_block_attn_bwd"):
        getattr(lib, name).restype = I
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(status, where):
    if status != USP_OK:
        raise UspError(status, where)


def problem(bs, L, hc, hk, hs, ulysses, ring, causal, split=USP_SPLIT_ZIGZAG, dtype=USP_BF16, scale=0.0):
    return usp_problem(bs, L, hc, hk, hs, ulysses, ring, int(bool(causal)), split, dtype, scale)


def usp_status_str(status):
    return load().usp_status_str(int(status)).decode()


def usp_validate(p):
    return load().usp_validate(C.byref(p))


def usp_local_positions(p, ring_rank, ulysses_rank):
    """Returns (shard, ring_block) position descriptors of virtual rank (ring_rank, ulysses_rank)."""
    shard, blk = usp_posdesc(), usp_posdesc()
    _check(load().usp_local_positions(C.byref(p), ring_rank, ulysses_rank, C.byref(shard), C.byref(blk)),
           "usp_local_positions")
    return shard, blk


def usp_layout_a2a(p, heads, direction, src, dst, rank_begin, rank_end, stream=None):
    _check(load().usp_layout_a2a(C.byref(p), heads, direction, _ptr(src), _ptr(dst), rank_begin, rank_end,
                                 _stream(stream)), "usp_layout_a2a")


def usp_block_attn_fwd(q, k, v, o_part, lse_part, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos, kpos, in_dtype,
                       o_dtype, stream=None):
    _check(load().usp_block_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o_part), _ptr(lse_part), bs, Lq, Lk, hq, hkv, hs,
                                     scale, int(bool(causal)), C.byref(qpos) if qpos is not None else None,
                                     C.byref(kpos) if kpos is not None else None, in_dtype, o_dtype, _stream(stream)),
           "usp_block_attn_fwd")


def usp_block_attn_fwd_state_bytes(bs, Lq, hq, hs):
    return int(load().usp_block_attn_fwd_state_bytes(bs, Lq, hq, hs))


def usp_block_attn_fwd_state(q, k, v, state, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos, kpos, first, last,
                             o_dtype, stream=None):
    _check(load().usp_block_attn_fwd_state(_ptr(q), _ptr(k), _ptr(v), _ptr(state), state.numel() * state.element_size(),
                                           _ptr(o), _ptr(lse), bs, Lq, Lk, hq, hkv, hs, scale, int(bool(causal)),
                                           C.byref(qpos) if qpos is not None else None,
                                           C.byref(kpos) if kpos is not None else None, int(bool(first)),
                                           int(bool(last)), o_dtype, _stream(stream)), "usp_block_attn_fwd_state")


def usp_lse_merge(o_parts, lse_parts, o_out, lse_out, bs, Lq, hq, hs, part_dtype, out_dtype, stream=None):
    n = len(o_parts)
    oa = (C.c_void_p * n)(*[_ptr(x) for x in o_parts])
    la = (C.c_void_p * n)(*[_ptr(x) for x in lse_parts])
    _check(load().usp_lse_merge(oa, la, n, _ptr(o_out), _ptr(lse_out), bs, Lq, hq, hs, part_dtype, out_dtype,
                                _stream(stream)), "usp_lse_merge")


def usp_ring_attn_fwd(q, k_blocks, v_blocks, kpos_blocks, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos,
                      in_dtype, o_dtype, stream=None):
    n = len(k_blocks)
    ka = (C.c_void_p * n)(*[_ptr(x) for x in k_blocks])
    va = (C.c_void_p * n)(*[_ptr(x) for x in v_blocks])
    kd = (usp_posdesc * n)(*kpos_blocks) if kpos_blocks is not None else None
    _check(load().usp_ring_attn_fwd(_ptr(q), ka, va, kd, n, _ptr(o), _ptr(lse), bs, Lq, Lk, hq, hkv, hs, scale,
                                    int(bool(causal)), C.byref(qpos) if qpos is not None else None, in_dtype,
                                    o_dtype, _stream(stream)), "usp_ring_attn_fwd")


def usp_ring_attn_fwd_vt(q, k_blocks, vt_blocks, kpos_blocks, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos,
                         stream=None):
    n = len(k_blocks)
    ka = (C.c_void_p * n)(*[_ptr(x) for x in k_blocks])
    va = (C.c_void_p * n)(*[_ptr(x) for x in vt_blocks])
    kd = (usp_posdesc * n)(*kpos_blocks) if kpos_blocks is not None else None
    _check(load().usp_ring_attn_fwd_vt(_ptr(q), ka, va, kd, n, _ptr(o), _ptr(lse), bs, Lq, Lk, hq, hkv, hs, scale,
                                       int(bool(causal)), C.byref(qpos) if qpos is not None else None,
                                       _stream(stream)), "usp_ring_attn_fwd_vt")


def usp_ring_attn_fwd_partials(q, k_blocks, v_blocks, kpos_blocks, lk_blocks, o_parts, lse_parts, bs, Lq, Lk, hq, hkv,
                               hs, scale, causal, qpos, stream=None):
    """k_blocks / v_blocks: tensors, or integer device addresses (pieces of one tensor)."""
    n = len(k_blocks)
    ka = (C.c_void_p * n)(*[_ptr(x) for x in k_blocks])
    va = (C.c_void_p * n)(*[_ptr(x) for x in v_blocks])
    kd = (usp_posdesc * n)(*kpos_blocks) if kpos_blocks is not None else None
    lk = (C.c_int32 * n)(*lk_blocks) if lk_blocks is not None else None
    oa = (C.c_void_p * n)(*[_ptr(x) for x in o_parts])
    la = (C.c_void_p * n)(*[_ptr(x) for x in lse_parts])
    _check(load().usp_ring_attn_fwd_partials(_ptr(q), ka, va, kd, lk, n, oa, la, bs, Lq, Lk, hq, hkv, hs, scale,
                                             int(bool(causal)), C.byref(qpos) if qpos is not None else None,
                                             _stream(stream)), "usp_ring_attn_fwd_partials")


def usp_attn_fwd_workspace_bytes(p, n_ranks):
    return int(load().usp_attn_fwd_workspace_bytes(C.byref(p), n_ranks))


def usp_attn_fwd(p, q, k, v, o, lse, rank_begin, rank_end, workspace, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(load().usp_attn_fwd(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), rank_begin, rank_end,
                               _ptr(workspace), workspace_bytes, _stream(stream)), "usp_attn_fwd")


USP_NOALLOC_SCRATCH_BYTES = 128 << 20


def usp_attn_fwd_noalloc(p, q, k, v, o, lse, rank_begin, rank_end, stream=None):
    _check(load().usp_attn_fwd_noalloc(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), rank_begin, rank_end,
                                       _stream(stream)), "usp_attn_fwd_noalloc")


def usp_attn_delta(o, d_o, delta, bs, L, h, hs, stream=None):
    _check(load().usp_attn_delta(_ptr(o), _ptr(d_o), _ptr(delta), bs, L, h, hs, _stream(stream)), "usp_attn_delta")


def usp_block_attn_bwd(q, k, v, d_o, lse, delta, dq, dk, dv, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos, kpos,
                       accumulate, stream=None):
    _check(load().usp_block_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta), _ptr(dq), _ptr(dk),
                                     _ptr(dv), bs, Lq, Lk, hq, hkv, hs, scale, int(bool(causal)),
                                     C.byref(qpos) if qpos is not None else None,
                                     C.byref(kpos) if kpos is not None else None, int(bool(accumulate)),
                                     _stream(stream)), "usp_block_attn_bwd")


def usp_ring_attn_bwd(q, k_blocks, v_blocks, kpos_blocks, d_o, lse, delta, dq, dk_blocks, dv_blocks, bs, Lq, Lk, hq, hkv,
                      hs, scale, causal, qpos, accumulate_dq, accumulate_dkdv, stream=None):
    n = len(k_blocks)
    arr = lambda xs: (C.c_void_p * n)(*[_ptr(x) for x in xs])
    kd = (usp_posdesc * n)(*kpos_blocks) if kpos_blocks is not None else None
    acc = (C.c_int * n)(*[int(bool(x)) for x in accumulate_dkdv])
    _check(load().usp_ring_attn_bwd(_ptr(q), arr(k_blocks), arr(v_blocks), kd, n, _ptr(d_o), _ptr(lse), _ptr(delta),
                                    _ptr(dq), arr(dk_blocks), arr(dv_blocks), bs, Lq, Lk, hq, hkv, hs, scale,
                                    int(bool(causal)), C.byref(qpos) if qpos is not None else None,
                                    int(bool(accumulate_dq)), acc, _stream(stream)), "usp_ring_attn_bwd")


def usp_ring_attn_bwd_workspace_bytes(bs, Lq, Lk, hq, hkv, hs, n_blocks):
    return int(load().usp_ring_attn_bwd_workspace_bytes(bs, Lq, Lk, hq, hkv, hs, n_blocks))


def usp_ring_attn_bwd_workspace_bytes_with_ds(bs, Lq, Lk, hq, hkv, hs, n_blocks):
    return int(load().usp_ring_attn_bwd_workspace_bytes_with_ds(bs, Lq, Lk, hq, hkv, hs, n_blocks))


def usp_ring_attn_bwd_ws(q, k_blocks, v_blocks, kpos_blocks, d_o, lse, delta, dq, dk_blocks, dv_blocks, bs, Lq, Lk, hq,
                         hkv, hs, scale, causal, qpos, accumulate_dq, accumulate_dkdv, workspace, workspace_bytes=None,
                         stream=None):
    n = len(k_blocks)
    arr = lambda xs: (C.c_void_p * n)(*[_ptr(x) for x in xs])
    kd = (usp_posdesc * n)(*kpos_blocks) if kpos_blocks is not None else None
    acc = (C.c_int * n)(*[int(bool(x)) for x in accumulate_dkdv])
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().usp_ring_attn_bwd_ws(_ptr(q), arr(k_blocks), arr(v_blocks), kd, n, _ptr(d_o), _ptr(lse), _ptr(delta),
                                       _ptr(dq), arr(dk_blocks), arr(dv_blocks), bs, Lq, Lk, hq, hkv, hs, scale,
                                       int(bool(causal)), C.byref(qpos) if qpos is not None else None,
                                       int(bool(accumulate_dq)), acc, _ptr(workspace), workspace_bytes,
                                       _stream(stream)), "usp_ring_attn_bwd_ws")


def usp_attn_bwd_workspace_bytes(p, n_ranks):
    return int(load().usp_attn_bwd_workspace_bytes(C.byref(p), n_ranks))


def usp_attn_bwd_workspace_bytes_with_ds(p, n_ranks):
    return int(load().usp_attn_bwd_workspace_bytes_with_ds(C.byref(p), n_ranks))


def usp_attn_bwd(p, q, k, v, o, lse, d_o, dq, dk, dv, rank_begin, rank_end, workspace, workspace_bytes=None,
                 stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(load().usp_attn_bwd(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq),
                               _ptr(dk), _ptr(dv), rank_begin, rank_end, _ptr(workspace), workspace_bytes,
                               _stream(stream)), "usp_attn_bwd")
