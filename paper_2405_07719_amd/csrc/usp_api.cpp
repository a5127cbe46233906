// C-ABI entry points: host-side validation, Algorithm 2 index arithmetic, and the
// orchestration of Algorithm 1 (all-to-all -> ring loop -> merge -> all-to-all) over kernels.
// No arithmetic of the method runs on the host; every step is a kernel launch.
#include <math.h>

#include <algorithm>
#include <functional>
#include <mutex>
#include <string.h>
#include <vector>

#include "usp_internal.h"

using namespace usp;

extern "C" const char* usp_status_str(int s) {
  switch (s) {
    case USP_OK: return "ok";
    case USP_ERR_NULL: return "null pointer";
    case USP_ERR_SHAPE: return "bad shape (sizes must be positive; L must divide by N, or by 2*R*U for the zigzag split)";
    case USP_ERR_DEGREE: return "bad degree (need U,R >= 1, hc % U == 0, hk % U == 0, hc % hk == 0)";
    case USP_ERR_DTYPE: return "bad dtype";
    case USP_ERR_WORKSPACE: return "workspace missing or too small";
    case USP_ERR_UNSUPPORTED: return "unsupported configuration";
    case USP_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

extern "C" int usp_validate(const usp_problem* p) {
  if (!p) return USP_ERR_NULL;
  if (p->bs < 1 || p->L < 1 || p->hc < 1 || p->hk < 1 || p->hs < 1) return USP_ERR_SHAPE;
  if (p->ulysses < 1 || p->ring < 1) return USP_ERR_DEGREE;
  if (p->hc % p->hk) return USP_ERR_DEGREE;
  // Sec. 3: the Ulysses degree is limited by the (KV) head count.
  if (p->hc % p->ulysses || p->hk % p->ulysses) return USP_ERR_DEGREE;
  if (p->dtype != USP_BF16 && p->dtype != USP_FP32) return USP_ERR_DTYPE;
  if (p->split != USP_SPLIT_CONTIG && p->split != USP_SPLIT_ZIGZAG) return USP_ERR_UNSUPPORTED;
  const int64_t n = (int64_t)p->ulysses * p->ring;
  if (p->split == USP_SPLIT_ZIGZAG) {
    if (p->L % (2 * n)) return USP_ERR_SHAPE;
  } else if (p->L % n) {
    return USP_ERR_SHAPE;
  }
  if (p->hs != 64 && p->hs != 128) return USP_ERR_UNSUPPORTED;
  if (p->L >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  if (!(p->scale >= 0.0f) || isinf(p->scale)) return USP_ERR_UNSUPPORTED;
  return USP_OK;
}

// Algorithm 2: ring rank r owns chunks r and 2R-1-r (of 2R); Ulysses rank u the u-th of U pieces.
static void ring_block_desc(const usp_problem& p, int r, usp_posdesc* d) {
  if (p.split == USP_SPLIT_ZIGZAG) {
    const int64_t c = p.L / (2 * (int64_t)p.ring);
    d->start0 = (int64_t)r * c;
    d->len0 = c;
    d->start1 = (2 * (int64_t)p.ring - 1 - r) * c;
    d->len1 = c;
  } else {
    const int64_t n = p.L / p.ring;
    d->start0 = (int64_t)r * n;
    d->len0 = n;
    d->start1 = d->start0 + n;
    d->len1 = 0;
  }
}

extern "C" int usp_local_positions(const usp_problem* p, int ring_rank, int ulysses_rank, usp_posdesc* shard,
                                   usp_posdesc* ring_block) {
  int st = usp_validate(p);
  if (st != USP_OK) return st;
  if (ring_rank < 0 || ring_rank >= p->ring || ulysses_rank < 0 || ulysses_rank >= p->ulysses)
    return USP_ERR_UNSUPPORTED;
  usp_posdesc blk;
  ring_block_desc(*p, ring_rank, &blk);
  if (ring_block) *ring_block = blk;
  if (shard) {
    // local indices [a, b) of the ring block, cut against the block's two runs
    const int64_t n = (blk.len0 + blk.len1) / p->ulysses;
    const int64_t a = (int64_t)ulysses_rank * n, b = a + n;
    const int64_t a0 = a < blk.len0 ? a : blk.len0, b0 = b < blk.len0 ? b : blk.len0;   // part in run 0
    const int64_t a1 = (a > blk.len0 ? a : blk.len0) - blk.len0, b1 = (b > blk.len0 ? b : blk.len0) - blk.len0;
    shard->start0 = blk.start0 + a0;
    shard->len0 = b0 - a0;
    shard->start1 = blk.start1 + a1;
    shard->len1 = b1 - a1;
  }
  return USP_OK;
}

extern "C" int usp_layout_a2a(const usp_problem* p, int heads, int dir, const void* src, void* dst, int rank_begin,
                              int rank_end, void* stream) {
  int st = usp_validate(p);
  if (st != USP_OK) return st;
  if (!src || !dst) return USP_ERR_NULL;
  if (heads < 1 || heads % p->ulysses) return USP_ERR_DEGREE;
  if (dir != USP_SEQ_TO_HEAD && dir != USP_HEAD_TO_SEQ && dir != USP_SEQ_TO_HEAD_VT) return USP_ERR_UNSUPPORTED;
  const int n = p->ulysses * p->ring;
  if (rank_begin < 0 || rank_end > n || rank_begin > rank_end) return USP_ERR_UNSUPPORTED;
  if (dir == USP_SEQ_TO_HEAD_VT && p->dtype != USP_BF16) return USP_ERR_DTYPE;
  if (rank_begin == rank_end) return USP_OK;
  if (dir == USP_SEQ_TO_HEAD_VT)
    return launch_layout_a2a_vt(*p, heads, src, dst, rank_begin, rank_end, 0, (hipStream_t)stream);
  return launch_layout_a2a(*p, heads, dir, src, dst, rank_begin, rank_end, 0, (hipStream_t)stream);
}

static bool desc_ok(const usp_posdesc* d, int64_t len) {
  // positions must fit 32 bits: the kernels narrow them
  const int64_t lim = (int64_t)1 << 31;
  return d && d->len0 >= 0 && d->len1 >= 0 && d->len0 + d->len1 == len && d->start0 >= 0 && d->start1 >= 0 &&
         d->start0 + d->len0 < lim && d->start1 + d->len1 < lim;
}

extern "C" int usp_block_attn_fwd(const void* q, const void* k, const void* v, void* o_part, float* lse_part, int bs,
                                  int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                                  const usp_posdesc* qpos, const usp_posdesc* kpos, int in_dtype, int o_dtype,
                                  void* stream) {
  if (!q || !k || !v || !o_part || !lse_part) return USP_ERR_NULL;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if ((in_dtype != USP_BF16 && in_dtype != USP_FP32) || (o_dtype != USP_BF16 && o_dtype != USP_FP32))
    return USP_ERR_DTYPE;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  usp_posdesc qd = {0, Lq, 0, 0}, kd = {0, Lk, 0, 0};
  if (causal) {
    if (!qpos || !kpos) return USP_ERR_NULL;
    if (!desc_ok(qpos, Lq) || !desc_ok(kpos, Lk)) return USP_ERR_SHAPE;
    qd = *qpos;
    kd = *kpos;
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  return launch_block_attn_fwd(q, k, v, o_part, lse_part, bs, Lq, Lk, hq, hkv, hs, scale, causal ? 1 : 0, qd, kd,
                               in_dtype, o_dtype, (hipStream_t)stream);
}

extern "C" size_t usp_block_attn_fwd_state_bytes(int bs, int64_t Lq, int hq, int hs) {
  if (bs < 1 || Lq < 1 || hq < 1 || (hs != 64 && hs != 128) || Lq >= (int64_t)1 << 31) return 0;
  return attn_fwd_state_bytes(bs, Lq, hq, hs);
}

extern "C" int usp_block_attn_fwd_state(const void* q, const void* k, const void* v, void* state, size_t state_bytes,
                                        void* o, float* lse, int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                                        float scale, int causal, const usp_posdesc* qpos, const usp_posdesc* kpos,
                                        int first, int last, int o_dtype, void* stream) {
  if (!q || !k || !v || !state) return USP_ERR_NULL;
  if (last && (!o || !lse)) return USP_ERR_NULL;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (o_dtype != USP_BF16 && o_dtype != USP_FP32) return USP_ERR_DTYPE;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  if (state_bytes < attn_fwd_state_bytes(bs, Lq, hq, hs) || ((uintptr_t)state & 15)) return USP_ERR_WORKSPACE;
  usp_posdesc qd = {0, Lq, 0, 0}, kd = {0, Lk, 0, 0};
  if (causal) {
    if (!qpos || !kpos) return USP_ERR_NULL;
    if (!desc_ok(qpos, Lq) || !desc_ok(kpos, Lk)) return USP_ERR_SHAPE;
    qd = *qpos;
    kd = *kpos;
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  const RingState rs = {(float*)state, first ? 1 : 0, last ? 1 : 0};
  return launch_ring_attn_fwd(q, &k, &v, &kd, 1, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal ? 1 : 0, qd, USP_BF16,
                              o_dtype, (hipStream_t)stream, nullptr, &rs);
}

namespace {
int ring_attn_fwd_impl(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                       const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                       int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                       int in_dtype, int o_dtype, void* stream, bool v_transposed);
}  // namespace

extern "C" int usp_ring_attn_fwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                                 const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                                 int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                                 int in_dtype, int o_dtype, void* stream) {
  return ring_attn_fwd_impl(q, k_blocks, v_blocks, kpos_blocks, n_blocks, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal,
                            qpos, in_dtype, o_dtype, stream, false);
}

extern "C" int usp_ring_attn_fwd_vt(const void* q, const void* const* k_blocks, const void* const* vt_blocks,
                                    const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs,
                                    int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                                    const usp_posdesc* qpos, void* stream) {
  return ring_attn_fwd_impl(q, k_blocks, vt_blocks, kpos_blocks, n_blocks, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal,
                            qpos, USP_BF16, USP_BF16, stream, true);
}

namespace {
int ring_attn_fwd_impl(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                       const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                       int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                       int in_dtype, int o_dtype, void* stream, bool v_transposed) {
  if (!q || !k_blocks || !v_blocks || !o || !lse) return USP_ERR_NULL;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return USP_ERR_UNSUPPORTED;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (in_dtype != USP_BF16 || (o_dtype != USP_BF16 && o_dtype != USP_FP32)) return USP_ERR_DTYPE;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  usp_posdesc qd = {0, Lq, 0, 0};
  usp_posdesc kd[USP_MAX_RING_BLOCKS];
  if (causal && (!qpos || !kpos_blocks)) return USP_ERR_NULL;
  if (causal && !desc_ok(qpos, Lq)) return USP_ERR_SHAPE;
  if (causal) qd = *qpos;
  for (int j = 0; j < n_blocks; ++j) {
    if (!k_blocks[j] || !v_blocks[j]) return USP_ERR_NULL;
    kd[j] = usp_posdesc{0, Lk, 0, 0};
    if (causal) {
      if (!desc_ok(&kpos_blocks[j], Lk)) return USP_ERR_SHAPE;
      kd[j] = kpos_blocks[j];
    }
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  if (v_transposed)
    for (int j = 0; j < n_blocks; ++j)
      if ((uintptr_t)v_blocks[j] & 15) return USP_ERR_UNSUPPORTED;
  return launch_ring_attn_fwd(q, k_blocks, v_blocks, kd, n_blocks, o, lse, bs, Lq, Lk, hq, hkv, hs, scale,
                              causal ? 1 : 0, qd, in_dtype, o_dtype, (hipStream_t)stream, nullptr, nullptr, v_transposed);
}
}  // namespace

extern "C" int usp_ring_attn_fwd_partials(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                                          const usp_posdesc* kpos_blocks, const int32_t* lk_blocks, int n_blocks,
                                          float* const* o_parts, float* const* lse_parts, int bs, int64_t Lq,
                                          int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                                          const usp_posdesc* qpos, void* stream) {
  if (!q || !k_blocks || !v_blocks || !o_parts || !lse_parts) return USP_ERR_NULL;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return USP_ERR_UNSUPPORTED;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  usp_posdesc qd = {0, Lq, 0, 0};
  usp_posdesc kd[USP_MAX_RING_BLOCKS];
  int lk[USP_MAX_RING_BLOCKS];
  if (causal && (!qpos || !kpos_blocks)) return USP_ERR_NULL;
  if (causal && !desc_ok(qpos, Lq)) return USP_ERR_SHAPE;
  if (causal) qd = *qpos;
  for (int j = 0; j < n_blocks; ++j) {
    if (!k_blocks[j] || !v_blocks[j] || !o_parts[j] || !lse_parts[j]) return USP_ERR_NULL;
    lk[j] = lk_blocks ? lk_blocks[j] : (int)Lk;
    if (lk[j] < 1 || lk[j] > Lk) return USP_ERR_SHAPE;
    kd[j] = usp_posdesc{0, lk[j], 0, 0};
    if (causal) {
      if (!desc_ok(&kpos_blocks[j], lk[j])) return USP_ERR_SHAPE;
      kd[j] = kpos_blocks[j];
    }
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  return launch_attn_fwd_partials(q, k_blocks, v_blocks, kd, lk, n_blocks, o_parts, lse_parts, bs, Lq, Lk, hq, hkv, hs,
                                  scale, causal ? 1 : 0, qd, (hipStream_t)stream);
}

extern "C" int usp_lse_merge(const void* const* o_parts, const float* const* lse_parts, int n_parts, void* o_out,
                             float* lse_out, int bs, int64_t Lq, int hq, int hs, int part_dtype, int out_dtype,
                             void* stream) {
  if (!o_parts || !lse_parts || !o_out || !lse_out) return USP_ERR_NULL;
  if (n_parts < 1 || n_parts > USP_MAX_MERGE_PARTS) return USP_ERR_UNSUPPORTED;
  for (int i = 0; i < n_parts; ++i)
    if (!o_parts[i] || !lse_parts[i]) return USP_ERR_NULL;
  if (bs < 1 || Lq < 1 || hq < 1 || hs < 1) return USP_ERR_SHAPE;
  if (hs % 8) return USP_ERR_UNSUPPORTED;
  if ((part_dtype != USP_BF16 && part_dtype != USP_FP32) || (out_dtype != USP_BF16 && out_dtype != USP_FP32))
    return USP_ERR_DTYPE;
  // An output may be the very buffer of a part only where the kernel is in-place safe: same element size (a thread
  // overwrites exactly the bytes it has read) and a row's threads inside one wavefront (hs / 4 divides 64), so that
  // the row's reads of the part's LSE precede the one store to it.  Any other overlap would read overwritten data.
  {
    const size_t rows = (size_t)bs * (size_t)Lq * hq;
    const size_t ob = rows * hs * dtype_size(out_dtype), pb = rows * hs * dtype_size(part_dtype), lb = rows * sizeof(float);
    const bool in_place_ok = part_dtype == out_dtype && (hs == 64 || hs == 128);
    auto overlap = [](const void* a, size_t na, const void* b, size_t nb) {
      return (const char*)a < (const char*)b + nb && (const char*)b < (const char*)a + na;
    };
    for (int i = 0; i < n_parts; ++i) {
      if (overlap(o_out, ob, o_parts[i], pb) && !(in_place_ok && o_out == o_parts[i])) return USP_ERR_UNSUPPORTED;
      if (overlap(lse_out, lb, lse_parts[i], lb) && !(in_place_ok && lse_out == lse_parts[i])) return USP_ERR_UNSUPPORTED;
      if (overlap(o_out, ob, lse_parts[i], lb) || overlap(lse_out, lb, o_parts[i], pb)) return USP_ERR_UNSUPPORTED;
    }
  }
  return launch_lse_merge(o_parts, lse_parts, n_parts, o_out, lse_out, bs, Lq, hq, hs, part_dtype, out_dtype,
                          (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1 forward.  Workspace plan (all sizes rounded up to 256 B):
//   kv_head : K and V in head layout for every (ring row, Ulysses column in range): the ring loop of
//             a rank reads block s = (r - i) mod R of its own column u;
//   q_head, o_head : one rank's Q / O in head layout (reused rank after rank, stream-ordered); only on the
//             step-by-step path (the one-launch ring loop reads and writes the sequence-layout shards itself);
//   parts   : R partial O (fp32) + R partial LSE when R > 1.
// ---------------------------------------------------------------------------------------------
namespace {

inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

struct FwdPlan {
  size_t q_head, o_head, k_head, v_head, o_parts, lse_parts, total;
  size_t kv_block_bytes, v_block_bytes, part_o_bytes, part_lse_bytes;
  int n_cols;
  bool v_transposed;   // V blocks are staged in key-tile-transposed layout (the one-launch ring loop reads them so)
  // Ulysses degree 1: a K/V block in head layout IS its sequence-layout shard.  K is then never staged; V only when it
  // is wanted in transposed tiles and re-tiling it costs less than the tiles save.
  bool k_in_place, v_in_place;
};

// Ulysses columns touched by ranks [rb, re): all U when the range spans more than one ring row.
void column_range(const usp_problem& p, int rb, int re, int* c0, int* c1) {
  const int U = p.ulysses;
  if (re - rb >= U || (rb / U) != ((re - 1) / U)) {
    *c0 = 0;
    *c1 = U;
  } else {
    *c0 = rb % U;
    *c1 = (re - 1) % U + 1;
  }
}

// The ring loop of a rank runs as one launch (state in registers, no partials, no merge) when the kernel family
// supports it: bf16 data and few enough blocks for the launch arguments.
bool ring_in_one_launch(const usp_problem& p) { return p.dtype == USP_BF16 && p.ring <= USP_MAX_RING_BLOCKS; }

// Key split of a rank's ring loop (launch_attn_fwd_partials): 0 = none (one work item per query tile, head and
// batch walks all blocks), else the number of pieces each K/V block is cut into, every piece of every block then
// being a work item of its own with a partial result of its own (1: the blocks themselves, for R > 1).  In the
// unsplit launch the item of the last query tile walks every key, which takes ratio = 256 / (items x 1/2 under
// a causal mask) times a CU's fair share of the whole launch.  Split from a ratio of 1.5: into two parts in all, three
// from a ratio of 3.5, four from 7 (the R blocks as they are when that is already as many or more); more parts cost
// more in partial results (fp32, written and merged) than they gain, and with one or two items per CU the finish time
// is a bin-packing matter (measured at L = 8192 and 16384: 2 and 3 pieces 1.4-1.8 x faster than none, 4 and more slower
// again; at L = 4096: 76 / 64 / 58 us with 2 / 3 / 4).  Pieces hold at least 1024 keys, and a launch takes no more parts in
// all than it takes blocks.  Host arithmetic only, with the chip's CU count as a constant (kPlanCUs): the workspace
// query must not need a GPU.
int key_splits(const usp_problem& p) {
  if (!ring_in_one_launch(p)) return 0;
  const int64_t Lq = p.L / p.ring;
  const int64_t items = ((Lq + 255) / 256) * (p.hc / p.ulysses) * p.bs;
  const double ratio = (double)kPlanCUs / ((double)items * (p.causal ? 0.5 : 1.0));
  if (ratio < 1.5) return 0;
  const int64_t parts_wanted = ratio >= 7.0 ? 4 : ratio >= 3.5 ? 3 : 2;
  int64_t s = (parts_wanted + p.ring - 1) / p.ring;
  s = std::min<int64_t>(s, Lq / 1024);
  s = std::min<int64_t>(s, USP_MAX_RING_BLOCKS / p.ring);
  s = std::max<int64_t>(s, 1);
  return s * p.ring > 1 ? (int)s : 0;
}

// Short of full grids (fewer than two work items per CU under a causal mask, the heaviest item longer than a CU's
// fair share) only the heaviest query tiles may be cut: the LAST `tiles` query tiles of the rank run as one item per
// piece of the keys (2 to 4 equal pieces of the one block when R = 1, else the R ring blocks), with fp32 partial results
// that are merged afterwards; the other tiles stay whole items of the same launch (launch_attn_fwd_partials with
// MixedLaunch).  How many tiles and pieces, if any, is decided by playing the launch through on the host: the kernel's
// own dealing (the first items given one per workgroup, the rest drawn in order by whoever is free), 8 us per item,
// 1.85 us per tile of 64 keys, 3 us each time a whole item moves on to another piece, and the merge of the cut rows at
// 5 TB/s + 10 us.  Host arithmetic only; the same for every Ulysses column of a ring row.
constexpr int kMaxHeavyPieces = USP_MAX_RING_BLOCKS;
struct HeavyPieces { int n; int64_t first[kMaxHeavyPieces], last[kMaxHeavyPieces]; int block[kMaxHeavyPieces]; };
struct HeavyChoice { int tiles, pieces; };   // tiles == 0: nothing is cut this way

// The pieces of a ring rank's keys, in the order its ring loop visits them: piece j = keys [first, last) of the block
// of ring step block[j].  R = 1: `pieces` equal parts of the one block (multiples of 64 keys); R > 1: the blocks.
HeavyPieces heavy_pieces(const usp_problem& p, int pieces) {
  HeavyPieces hp;
  const int64_t Lq = p.L / p.ring;
  if (p.ring == 1) {
    const int64_t piece = ((Lq + pieces - 1) / pieces + 63) / 64 * 64;
    hp.n = 0;
    for (int64_t a0 = 0; a0 < Lq; a0 += piece, ++hp.n) {
      hp.first[hp.n] = a0; hp.last[hp.n] = std::min(Lq, a0 + piece); hp.block[hp.n] = 0;
    }
  } else {
    hp.n = p.ring;
    for (int i = 0; i < p.ring; ++i) { hp.first[i] = 0; hp.last[i] = Lq; hp.block[i] = i; }
  }
  return hp;
}

// Positions of the keys [a, b) of a block whose positions are d.
usp_posdesc piece_of(const usp_posdesc& d, int64_t a, int64_t b) {
  if (a >= d.len0) return usp_posdesc{d.start1 + (a - d.len0), b - a, 0, 0};
  const int64_t n0 = std::min(b, d.len0) - a;
  return usp_posdesc{d.start0 + a, n0, d.start1, (b - a) - n0};
}

// What ring rank r cuts ({0, 0}: nothing, the launch is key_splits()' business).  (Worked out once per problem:
// heavy_choice() below keeps the answers.)
HeavyChoice work_out_heavy_choice(const usp_problem& p, int r) {
  const HeavyChoice none = {0, 0};
  if (!ring_in_one_launch(p)) return none;
  const int64_t Lq = p.L / p.ring;
  const int T = (int)((Lq + 255) / 256), n = (p.hc / p.ulysses) * p.bs;
  const int64_t items = (int64_t)T * n;
  if (items > 4 * kPlanCUs || Lq < 4096 || T < 8) return none;
  if (p.ring > 1 && items <= kPlanCUs) return none;   // short ring ranks: every tile per block, as key_splits() has it
  // Without a mask all items weigh the same and what is lost is the last, partly filled round (320 items on 256 CUs
  // take two rounds): the cut tiles' pieces then fill the first round and the whole items follow.
  if (!p.causal && items <= kPlanCUs) return none;
  usp_posdesc qd;
  ring_block_desc(p, r, &qd);
  const double kItem = 8.0, kTile = 1.85, kCross = 3.0;
  auto pos_of = [&](int64_t i) { return i < qd.len0 ? qd.start0 + i : qd.start1 + (i - qd.len0); };
  auto play = [&](const std::vector<double>& w) {
    std::vector<double> free_at;   // a min-heap of the workgroups' finish times
    free_at.reserve(kPlanCUs);
    size_t j = 0;
    for (; j < w.size() && (int)j < kPlanCUs; ++j) free_at.push_back(w[j]);
    std::make_heap(free_at.begin(), free_at.end(), std::greater<double>());
    for (; j < w.size(); ++j) {
      std::pop_heap(free_at.begin(), free_at.end(), std::greater<double>());
      free_at.back() += w[j];
      std::push_heap(free_at.begin(), free_at.end(), std::greater<double>());
    }
    double end = 0.0;
    for (double t : free_at) end = std::max(end, t);
    return end;
  };
  // time of the launch with the last k query tiles cut into the pieces hp (k = T: every tile, k = 0: none)
  auto launch_time = [&](const HeavyPieces& hp, int k) {
    // 64-key tiles of piece j that query tile i walks: under kpos <= qpos the visible keys of each run are a prefix of it
    std::vector<double> tiles((size_t)T * hp.n);
    for (int j = 0; j < hp.n; ++j) {
      usp_posdesc kd;
      ring_block_desc(p, ((r - hp.block[j]) % p.ring + p.ring) % p.ring, &kd);
      const usp_posdesc pd = piece_of(kd, hp.first[j], hp.last[j]);
      for (int i = 0; i < T; ++i) {
        const int64_t a = (int64_t)i * 256, b = std::min<int64_t>(Lq, a + 256);
        int64_t qmax = std::max(pos_of(a), pos_of(b - 1));
        if (a < qd.len0 && b > qd.len0) qmax = std::max({qmax, pos_of(qd.len0 - 1), pos_of(qd.len0)});
        const int64_t c0 = p.causal ? std::clamp<int64_t>(qmax - pd.start0 + 1, 0, pd.len0) : pd.len0;
        const int64_t c1 = p.causal ? std::clamp<int64_t>(qmax - pd.start1 + 1, 0, pd.len1) : pd.len1;
        tiles[(size_t)i * hp.n + j] = (double)((c0 + 63) / 64 + (c1 + 63) / 64);
      }
    }
    std::vector<double> w;
    w.reserve((size_t)items + (size_t)k * n * hp.n);
    for (int t = 0; t < k; ++t)
      for (int j = 0; j < hp.n; ++j)
        for (int h = 0; h < n; ++h) w.push_back(kItem + kTile * tiles[(size_t)(T - 1 - t) * hp.n + j]);
    for (int t = k; t < T; ++t) {
      double sum = 0.0;
      int walked = 0;
      for (int j = 0; j < hp.n; ++j) {
        sum += tiles[(size_t)(T - 1 - t) * hp.n + j];
        walked += tiles[(size_t)(T - 1 - t) * hp.n + j] > 0.0;
      }
      // (the one-launch ring loop pays the change of block too, so it is charged whether or not anything is cut)
      const double cross = (p.ring > 1 || k > 0) ? kCross * std::max(0, walked - 1) : 0.0;
      for (int h = 0; h < n; ++h) w.push_back(kItem + kTile * sum + cross);
    }
    double us = play(w);
    if (k > 0) {
      const double rows = (double)std::min<int64_t>(Lq, (int64_t)k * 256) * n;
      us += 10.0 + rows * p.hs * (hp.n * 2.0 * 4.0 + 2.0) / 5.0e6;   // the fp32 partials written and read, bf16 out
    }
    return us;
  };
  // what the launch costs as key_splits() has it: whole, or every tile in so many pieces per block
  const int splits = key_splits(p);
  const double as_is_us = splits > 0 ? launch_time(heavy_pieces(p, splits), T) : launch_time(heavy_pieces(p, 2), 0);
  // A cut has to pay for itself: 3 % by this model when the pieces are parts of one block and the launch was whole,
  // where the model's choice was the measured optimum at every length tried; 8 % when they are ring blocks of unequal
  // visible parts, where it promises 5 % more than is measured (the uncut launch's long tail runs on few CUs at a
  // higher clock); 5 % against a launch that already cuts every tile.
  const double need = p.ring > 1 ? 0.92 : splits > 0 ? 0.95 : 0.97;
  HeavyChoice best = none;
  double best_us = as_is_us;
  for (int pieces = 2; pieces <= (p.ring == 1 ? 4 : 2); ++pieces) {   // (R > 1: the blocks, one pass)
    if (p.ring == 1 && Lq / pieces < 1024) break;
    const HeavyPieces hp = heavy_pieces(p, pieces);
    for (int part = 1; part < 32; ++part) {   // k in steps of T / 32
      const int k = std::max(1, T * part / 32);
      if (part > 1 && k == std::max(1, T * (part - 1) / 32)) continue;
      const double us = launch_time(hp, k);
      if (us < best_us) { best = HeavyChoice{k, hp.n}; best_us = us; }
    }
  }
  if (best_us >= need * as_is_us) return none;
  return best;
}

// Playing a launch through takes the host 0.1-0.3 ms per ring rank, as long as a short launch itself: the answers
// for the last problems seen are kept (every ring rank's, worked out at the first question about the problem).
HeavyChoice heavy_choice(const usp_problem& p, int r) {
  struct Entry { usp_problem p; std::vector<HeavyChoice> per_rank; };
  static std::mutex mu;
  static std::vector<Entry> seen;
  auto same = [](const usp_problem& a, const usp_problem& b) {
    return a.bs == b.bs && a.L == b.L && a.hc == b.hc && a.hk == b.hk && a.hs == b.hs && a.ulysses == b.ulysses &&
           a.ring == b.ring && a.causal == b.causal && a.split == b.split && a.dtype == b.dtype;   // (the scale plays no part)
  };
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : seen)
    if (same(e.p, p)) return e.per_rank[r];
  if (seen.size() >= 64) seen.erase(seen.begin());
  Entry e{p, {}};
  for (int rr = 0; rr < p.ring; ++rr) e.per_rank.push_back(work_out_heavy_choice(p, rr));
  seen.push_back(e);
  return seen.back().per_rank[r];
}

// The most pieces any ring rank of the problem cuts its heaviest tiles into (0: no rank does): the workspace holds as
// many partial results.
int heavy_max_pieces(const usp_problem& p) {
  int m = 0;
  for (int r = 0; r < p.ring; ++r) {
    const HeavyChoice c = heavy_choice(p, r);
    if (c.tiles > 0) m = std::max(m, c.pieces);
  }
  return m;
}

// allow_heavy = false: as if no rank cut its heaviest tiles (the entry point without a workspace of its own falls back
// to that when the partials would not fit its array).
FwdPlan plan_fwd(const usp_problem& p, int n_cols, bool allow_heavy = true) {
  FwdPlan f;
  const size_t es = dtype_size(p.dtype);
  const size_t Lq = p.L / p.ring, hq = p.hc / p.ulysses, hkv = p.hk / p.ulysses;
  const size_t qb = up256((size_t)p.bs * Lq * hq * p.hs * es);
  f.kv_block_bytes = (size_t)p.bs * Lq * hkv * p.hs * es;   // exact: blocks are packed back to back (multiple of 128 B)
  f.part_o_bytes = up256((size_t)p.bs * Lq * hq * p.hs * sizeof(float));
  f.part_lse_bytes = up256((size_t)p.bs * Lq * hq * sizeof(float));
  f.n_cols = n_cols;
  size_t off = 0;
  // the one-launch ring loop reads Q from and writes O to the sequence-layout shards: no head-layout copies of them
  const size_t qo = ring_in_one_launch(p) ? 0 : qb;
  f.q_head = off; off += qo;
  f.o_head = off; off += qo;
  const int heavy = allow_heavy ? heavy_max_pieces(p) : 0;
  const int splits = key_splits(p);
  // The one-launch ring loop and the launch that cuts only the heaviest tiles (not the launch that cuts every tile,
  // whose fp32 instance reads V rows) take V in key-tile-transposed layout: tiles of 64 keys, the last one padded.
  // With Ulysses degree 1 the all-to-all of Algorithm 1 is the identity: block s in head layout, [bs][L/R][hk][hs], is
  // shard s as it stands, and the kernels read K where it is.  V too, as rows, unless re-tiling it (the only copy
  // left: all R blocks read and written at about 5 TB/s, one launch of about 6 us) costs less than the transposed
  // tiles save (1.3 % of the attention time, taken as visible pairs x 4 hs flop at 1.1 PFLOP/s).  Measured, one
  // ring-only rank of L = 32768, ring 8: 8 KV heads 1.014 -> 0.970 ms with both in place (0.987 estimated with V
  // re-tiled); one KV head 0.954 -> 0.960 ms with both in place, hence V re-tiled there.
  f.k_in_place = p.ulysses == 1;
  f.v_transposed = ring_in_one_launch(p) && splits == 0;
  if (f.k_in_place && f.v_transposed) {
    const double pairs = (double)p.bs * hq * (double)Lq * (double)p.L * (p.causal ? 0.5 : 1.0);
    const double attention_us = pairs * 4.0 * p.hs / 1.1e9;
    const double retile_us = 2.0 * (double)p.bs * p.L * hkv * p.hs * es / 5e6 + 6.0;
    if (retile_us > 0.013 * attention_us) f.v_transposed = false;
  }
  f.v_in_place = f.k_in_place && !f.v_transposed;
  f.v_block_bytes = f.v_transposed ? vt_block_bytes(p.bs, (int64_t)Lq, (int)hkv, p.hs) : f.kv_block_bytes;
  f.k_head = off; off += f.k_in_place ? 0 : up256(f.kv_block_bytes * p.ring * n_cols);
  f.v_head = off; off += f.v_in_place ? 0 : up256(f.v_block_bytes * p.ring * n_cols);
  size_t parts = splits > 0 ? (size_t)splits * p.ring : (p.ring > 1 && !ring_in_one_launch(p)) ? p.ring : 0;
  parts = std::max<size_t>(parts, (size_t)heavy);
  f.o_parts = off; off += f.part_o_bytes * parts;
  f.lse_parts = off; off += f.part_lse_bytes * parts;
  f.total = off;
  return f;
}

}  // namespace

namespace {

// K and V of every (ring row, Ulysses column in [c0, c1)) to head layout, packed by slot r * n_cols + (u - c0).
int stage_kv_blocks(const usp_problem& p, const void* k, const void* v, char* k_head, char* v_head, size_t block_bytes,
                    int c0, int c1, hipStream_t stream, size_t vt_block_bytes_ = 0) {
  const int U = p.ulysses, R = p.ring, n_cols = c1 - c0;
  if (vt_block_bytes_) {
    // K as rows, V in key-tile-transposed layout: one launch each, same ranks and slots
    int st = USP_OK;
    const void* ksrc[1] = {k};
    if (n_cols == U) {
      void* kdst[1] = {k_head};
      st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 1, ksrc, kdst, 0, U * R, -1, stream);
      if (st == USP_OK) st = launch_layout_a2a_vt(p, p.hk, v, v_head, 0, U * R, -1, stream);
    } else if (n_cols == 1) {
      void* kdst[1] = {k_head};
      st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 1, ksrc, kdst, c0, U * R, -1, stream, U);
      if (st == USP_OK) st = launch_layout_a2a_vt(p, p.hk, v, v_head, c0, U * R, -1, stream, U);
    } else {
      for (int r = 0; r < R && st == USP_OK; ++r) {
        void* kdst[1] = {k_head + (size_t)r * n_cols * block_bytes};
        st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 1, ksrc, kdst, r * U + c0, r * U + c1, -1, stream);
        if (st == USP_OK)
          st = launch_layout_a2a_vt(p, p.hk, v, v_head + (size_t)r * n_cols * vt_block_bytes_, r * U + c0, r * U + c1, -1, stream);
      }
    }
    return st;
  }
  // K and V have one geometry: both go through the same launches
  const void* src[2] = {k, v};
  int st = USP_OK;
  if (n_cols == U) {
    void* dst[2] = {k_head, v_head};
    st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 2, src, dst, 0, U * R, -1, stream);
  } else if (n_cols == 1) {
    void* dst[2] = {k_head, v_head};
    st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 2, src, dst, c0, U * R, -1, stream, U);
  } else {
    for (int r = 0; r < R && st == USP_OK; ++r) {
      void* dst[2] = {k_head + (size_t)r * n_cols * block_bytes, v_head + (size_t)r * n_cols * block_bytes};
      st = launch_layout_a2a_multi(p, p.hk, USP_SEQ_TO_HEAD, 2, src, dst, r * U + c0, r * U + c1, -1, stream);
    }
  }
  return st;
}

}  // namespace

extern "C" size_t usp_attn_fwd_workspace_bytes(const usp_problem* p, int n_ranks) {
  if (usp_validate(p) != USP_OK || n_ranks < 1) return 0;
  // one rank touches one Ulysses column; a wider range may straddle ring rows, so size for all U
  const int cols = n_ranks == 1 ? 1 : p->ulysses;
  return plan_fwd(*p, cols).total;
}

namespace {
int attn_fwd_impl(const usp_problem* p, const void* q, const void* k, const void* v, void* o, float* lse,
                  int rank_begin, int rank_end, void* workspace, size_t workspace_bytes, void* stream_,
                  bool allow_heavy = true) {
  int st = usp_validate(p);
  if (st != USP_OK) return st;
  if (!q || !k || !v || !o || !lse) return USP_ERR_NULL;
  const int U = p->ulysses, R = p->ring, N = U * R;
  if (rank_begin < 0 || rank_end > N || rank_begin >= rank_end) return USP_ERR_UNSUPPORTED;
  int c0, c1;
  column_range(*p, rank_begin, rank_end, &c0, &c1);
  const FwdPlan f = plan_fwd(*p, c1 - c0, allow_heavy);
  // (a plan that needs no workspace at all, as a ring-only problem in one launch, takes any pointer, null included)
  if (f.total > 0 && (!workspace || workspace_bytes < f.total || ((uintptr_t)workspace & 255))) return USP_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  char* ws = (char*)workspace;
  const size_t es = dtype_size(p->dtype);
  const int64_t Lq = p->L / R;
  const int hq = p->hc / U, hkv = p->hk / U;
  const float scale = p->scale == 0.0f ? 1.0f / sqrtf((float)p->hs) : p->scale;


  // Steps 3-4 of Algorithm 1 for every K/V block the ranks in range will visit.  The workspace slot of
  // block (r, u) is r * n_cols + (u - c0): with all U columns that is the rank order (one launch per
  // tensor); with one column the ranks r * U + u are a stride-U sequence (again one launch per tensor).
  const char* const k_blocks = f.k_in_place ? (const char*)k : ws + f.k_head;   // block slot 0 of K, of V
  const char* const v_blocks = f.v_in_place ? (const char*)v : ws + f.v_head;
  if (!f.k_in_place) {
    st = stage_kv_blocks(*p, k, v, ws + f.k_head, ws + f.v_head, f.kv_block_bytes, c0, c1, stream,
                         f.v_transposed ? f.v_block_bytes : 0);
    if (st != USP_OK) return st;
  } else if (!f.v_in_place) {
    // Ulysses degree 1, V wanted in transposed tiles: all R blocks in one launch, slot = ring row
    st = launch_layout_a2a_vt(*p, p->hk, v, ws + f.v_head, 0, R, -1, stream);
    if (st != USP_OK) return st;
  }

  for (int rank = rank_begin; rank < rank_end; ++rank) {
    const int r = rank / U, u = rank % U;
    // Step 2: Q of this rank to head layout (the one-launch ring loop reads the shards itself).
    if (!ring_in_one_launch(*p)) {
      st = launch_layout_a2a(*p, p->hc, USP_SEQ_TO_HEAD, q, ws + f.q_head, rank, rank + 1, rank, stream);
      if (st != USP_OK) return st;
    }
    usp_posdesc qd;
    usp_local_positions(p, r, u, nullptr, &qd);
    float* lse_rank = lse + (size_t)rank * p->bs * hq * Lq;
    // Step 5: the ring loop.  Step i visits block s = (r - i) mod R.
    if (ring_in_one_launch(*p)) {
      const void* kb[USP_MAX_RING_BLOCKS];
      const void* vb[USP_MAX_RING_BLOCKS];
      usp_posdesc kds[USP_MAX_RING_BLOCKS];
      for (int i = 0; i < R; ++i) {
        const int s = ((r - i) % R + R) % R;
        usp_local_positions(p, s, u, nullptr, &kds[i]);
        const size_t slot = (size_t)s * (c1 - c0) + (u - c0);
        kb[i] = k_blocks + slot * f.kv_block_bytes;
        vb[i] = v_blocks + slot * f.v_block_bytes;
      }
      // Steps 2 and 6 for Q and O ride on the kernel's own accesses: it reads each Q row once and writes each O
      // row once, so it does that straight from / to the sequence-layout shards of the Ulysses group.
      const SeqLayoutIO seq = {(int)(p->L / N), p->hc, u * hq};
      const size_t group_off = (size_t)r * U * p->bs * (p->L / N) * p->hc * p->hs * es;
      const HeavyChoice heavy = allow_heavy ? heavy_choice(*p, r) : HeavyChoice{0, 0};
      if (heavy.tiles > 0) {
        // Medium length: the last `heavy` query tiles as one item per piece of the keys (the halves of the one block, or
        // the ring blocks), with partial results; every other tile a whole item of the same launch that writes its
        // finished rows itself.  Then the merge of the cut rows, straight to the sequence-layout shards.
        const HeavyPieces hp = heavy_pieces(*p, heavy.pieces);
        const void* kp[kMaxHeavyPieces];
        const void* vp[kMaxHeavyPieces];
        usp_posdesc pd[kMaxHeavyPieces];
        int lk[kMaxHeavyPieces];
        float* o_ptrs[kMaxHeavyPieces];
        float* l_ptrs[kMaxHeavyPieces];
        for (int n = 0; n < hp.n; ++n) {
          const size_t row_off = (size_t)hp.first[n] * hkv * p->hs * es;
          kp[n] = (const char*)kb[hp.block[n]] + row_off;
          // (transposed tiles: a piece begins hp.first / 64 tiles into every head's run of tiles)
          vp[n] = (const char*)vb[hp.block[n]] + (f.v_transposed ? (size_t)(hp.first[n] / 64) * p->hs * 64 * es : row_off);
          pd[n] = piece_of(kds[hp.block[n]], hp.first[n], hp.last[n]);
          lk[n] = (int)(hp.last[n] - hp.first[n]);
          o_ptrs[n] = (float*)(ws + f.o_parts + (size_t)n * f.part_o_bytes);
          l_ptrs[n] = (float*)(ws + f.lse_parts + (size_t)n * f.part_lse_bytes);
        }
        const MixedLaunch mixed = {(char*)o + group_off, lse_rank, heavy.tiles, f.v_transposed};
        st = launch_attn_fwd_partials((const char*)q + group_off, kp, vp, pd, lk, hp.n, o_ptrs, l_ptrs, p->bs, Lq, Lq, hq,
                                      hkv, p->hs, scale, p->causal ? 1 : 0, qd, stream, &seq, &mixed);
        if (st != USP_OK) return st;
        const int64_t row0 = ((Lq + 255) / 256 - heavy.tiles) * 256;
        st = launch_lse_merge((const void* const*)o_ptrs, (const float* const*)l_ptrs, hp.n, (char*)o + group_off, lse_rank,
                              p->bs, Lq, hq, p->hs, USP_FP32, p->dtype, stream, &seq, row0);
        if (st != USP_OK) return st;
        continue;
      }
      const int splits = key_splits(*p);
      if (splits > 0) {
        // Short sequence: every block in `splits` pieces, each (query tile, head, piece) its own work item of one
        // launch; the pieces' partial results are merged, and O takes the separate pass back to the sequence layout.
        const int64_t piece = ((Lq + splits - 1) / splits + 63) / 64 * 64;
        const void* kp[USP_MAX_RING_BLOCKS];
        const void* vp[USP_MAX_RING_BLOCKS];
        usp_posdesc pd[USP_MAX_RING_BLOCKS];
        int lk[USP_MAX_RING_BLOCKS];
        float* o_ptrs[USP_MAX_RING_BLOCKS];
        float* l_ptrs[USP_MAX_RING_BLOCKS];
        int n = 0;
        for (int i = 0; i < R; ++i)
          for (int64_t a0 = 0; a0 < Lq; a0 += piece, ++n) {
            const int64_t a1 = std::min(Lq, a0 + piece);
            const size_t row_off = (size_t)a0 * hkv * p->hs * es;
            kp[n] = (const char*)kb[i] + row_off;
            vp[n] = (const char*)vb[i] + row_off;
            pd[n] = piece_of(kds[i], a0, a1);
            lk[n] = (int)(a1 - a0);
            o_ptrs[n] = (float*)(ws + f.o_parts + (size_t)n * f.part_o_bytes);
            l_ptrs[n] = (float*)(ws + f.lse_parts + (size_t)n * f.part_lse_bytes);
          }
        st = launch_attn_fwd_partials((const char*)q + group_off, kp, vp, pd, lk, n, o_ptrs, l_ptrs, p->bs, Lq, Lq, hq,
                                      hkv, p->hs, scale, p->causal ? 1 : 0, qd, stream, &seq);
        if (st != USP_OK) return st;
        // the merge writes O straight to the sequence-layout shards (step 6 rides on its stores)
        st = launch_lse_merge((const void* const*)o_ptrs, (const float* const*)l_ptrs, n, (char*)o + group_off, lse_rank,
                              p->bs, Lq, hq, p->hs, USP_FP32, p->dtype, stream, &seq);
        if (st != USP_OK) return st;
        continue;
      }
      st = launch_ring_attn_fwd((const char*)q + group_off, kb, vb, kds, R, (char*)o + group_off, lse_rank, p->bs, Lq,
                                Lq, hq, hkv, p->hs, scale, p->causal ? 1 : 0, qd, p->dtype, p->dtype, stream, &seq,
                                nullptr, f.v_transposed);
      if (st != USP_OK) return st;
      continue;
    }
    const void* o_ptrs[USP_MAX_MERGE_PARTS];
    const float* l_ptrs[USP_MAX_MERGE_PARTS];
    if (R > USP_MAX_MERGE_PARTS) return USP_ERR_UNSUPPORTED;
    for (int i = 0; i < R; ++i) {
      const int s = ((r - i) % R + R) % R;
      usp_posdesc kd;
      usp_local_positions(p, s, u, nullptr, &kd);
      const size_t slot = ((size_t)s * (c1 - c0) + (u - c0)) * f.kv_block_bytes;
      void* o_dst = R > 1 ? (void*)(ws + f.o_parts + (size_t)i * f.part_o_bytes) : (void*)(ws + f.o_head);
      float* l_dst = R > 1 ? (float*)(ws + f.lse_parts + (size_t)i * f.part_lse_bytes) : lse_rank;
      st = launch_block_attn_fwd(ws + f.q_head, k_blocks + slot, v_blocks + slot, o_dst, l_dst, p->bs, Lq,
                                 Lq, hq, hkv, p->hs, scale, p->causal ? 1 : 0, qd, kd, p->dtype,
                                 R > 1 ? USP_FP32 : p->dtype, stream);
      if (st != USP_OK) return st;
      o_ptrs[i] = o_dst;
      l_ptrs[i] = l_dst;
    }
    if (R > 1) {
      // Step 6 rides on the merge's stores: O goes straight to the sequence-layout shards of the Ulysses group
      const SeqLayoutIO seq = {(int)(p->L / N), p->hc, u * hq};
      const size_t group_off = (size_t)r * U * p->bs * (p->L / N) * p->hc * p->hs * es;
      st = launch_lse_merge(o_ptrs, l_ptrs, R, (char*)o + group_off, lse_rank, p->bs, Lq, hq, p->hs, USP_FP32, p->dtype,
                            stream, &seq);
      if (st != USP_OK) return st;
      continue;
    }
    // Step 6: O back to the sequence layout.
    st = launch_layout_a2a(*p, p->hc, USP_HEAD_TO_SEQ, ws + f.o_head, o, rank, rank + 1, rank, stream);
    if (st != USP_OK) return st;
  }
  return USP_OK;
}
}  // namespace

extern "C" int usp_attn_fwd(const usp_problem* p, const void* q, const void* k, const void* v, void* o, float* lse,
                            int rank_begin, int rank_end, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_fwd_impl(p, q, k, v, o, lse, rank_begin, rank_end, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// usp_attn_fwd for callers that cannot allocate: the workspace is a static device array.  Each GPU the library
// runs on holds its own copy of the array (at its own address) until the process ends; host code never uses the
// array's name as an address, only what hipGetSymbolAddress returned for the current device.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[USP_NOALLOC_SCRATCH_BYTES];

namespace {
// Device address of `scratch` on the current device (asked once per device), or null.
void* scratch_on_current_device() {
  static std::atomic<void*> known[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  void* ptr = known[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    known[dev].store(ptr, std::memory_order_release);   // two threads that meet here store the same address
  }
  return ptr;
}
}  // namespace

extern "C" int usp_attn_fwd_noalloc(const usp_problem* p, const void* q, const void* k, const void* v, void* o,
                                    float* lse, int rank_begin, int rank_end, void* stream) {
  int st = usp_validate(p);
  if (st != USP_OK) return st;
  const int N = p->ulysses * p->ring;
  if (rank_begin < 0 || rank_end > N || rank_begin >= rank_end) return USP_ERR_UNSUPPORTED;
  int c0, c1;
  column_range(*p, rank_begin, rank_end, &c0, &c1);
  // the partial results of a cut of the heaviest tiles are optional: without room for them the launch stays whole
  const bool heavy_fits = plan_fwd(*p, c1 - c0, true).total <= USP_NOALLOC_SCRATCH_BYTES;
  if (!heavy_fits && plan_fwd(*p, c1 - c0, false).total > USP_NOALLOC_SCRATCH_BYTES) return USP_ERR_WORKSPACE;   // beyond the static array
  void* ptr = scratch_on_current_device();
  if (!ptr) return USP_ERR_LAUNCH;
  // every region of the workspace is written by a kernel of the call before a kernel reads it: nothing to clear
  return attn_fwd_impl(p, q, k, v, o, lse, rank_begin, rank_end, ptr, USP_NOALLOC_SCRATCH_BYTES, stream, heavy_fits);
}

extern "C" int usp_attn_delta(const void* o, const void* d_o, float* delta, int bs, int64_t L, int h, int hs,
                              void* stream) {
  if (!o || !d_o || !delta) return USP_ERR_NULL;
  if (bs < 1 || L < 1 || h < 1) return USP_ERR_SHAPE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (L >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  return launch_bwd_delta(o, d_o, delta, bs, L, h, hs, (hipStream_t)stream);
}

extern "C" int usp_block_attn_bwd(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                                  const float* delta, float* dq, float* dk, float* dv, int bs, int64_t Lq, int64_t Lk,
                                  int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                                  const usp_posdesc* kpos, int accumulate, void* stream) {
  if (!q || !k || !v || !d_o || !lse || !delta || !dq || !dk || !dv) return USP_ERR_NULL;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  usp_posdesc qd = {0, Lq, 0, 0}, kd = {0, Lk, 0, 0};
  if (causal) {
    if (!qpos || !kpos) return USP_ERR_NULL;
    if (!desc_ok(qpos, Lq) || !desc_ok(kpos, Lk)) return USP_ERR_SHAPE;
    qd = *qpos;
    kd = *kpos;
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  return launch_block_attn_bwd(q, k, v, d_o, lse, delta, dq, dk, dv, bs, Lq, Lk, hq, hkv, hs, scale, causal ? 1 : 0,
                               qd, kd, accumulate ? 1 : 0, accumulate ? 1 : 0, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// Algorithm 1 backward.  Workspace plan:
//   q_head, do_head         : one rank's Q and dO in head layout (reused rank after rank); O is read once, for D_i,
//                             straight from the sequence-layout shards;
//   (with Ulysses degree 1 a rank's Q, dO and every K/V block in head layout ARE the sequence-layout shards: these
//   four regions are empty and the kernels read the caller's tensors where they are)
//   delta                   : one rank's D_i;
//   k_head, v_head          : as in the forward; later hold the converted dK / dV blocks;
//   dq_acc                  : one rank's fp32 dQ;  dk_acc, dv_acc : fp32, one per K/V block.
// ---------------------------------------------------------------------------------------------
namespace {

struct BwdPlan {
  size_t q_head, do_head, delta, k_head, v_head, dq_acc, dk_acc, dv_acc, total;
  size_t kv_block_bytes, kv_acc_bytes;   // kv_acc_bytes: ALL copies of one block's dk (or dv) accumulator
  BwdCopies copies;                      // how the launch pairs are cut, and the copies of dq / dk / dv they fill
  int dkdv_copies;
  size_t ds, ds_bytes;                   // room for the dS of one launch pair (used when the workspace reaches that far)
  size_t total_with_ds;
};

BwdPlan plan_bwd(const usp_problem& p, int n_cols) {
  BwdPlan f;
  const size_t es = dtype_size(p.dtype);
  const size_t Lq = p.L / p.ring, hq = p.hc / p.ulysses, hkv = p.hk / p.ulysses;
  const size_t q_elems = (size_t)p.bs * Lq * hq * p.hs, kv_elems = (size_t)p.bs * Lq * hkv * p.hs;
  const size_t qb = up256(q_elems * es);
  f.kv_block_bytes = kv_elems * es;   // exact: blocks are packed back to back
  // every launch pair of this problem is cut the same way (that of its largest launch: up to 16 blocks)
  f.copies.cut = plan_bwd_cut(p.bs, (int64_t)Lq, (int64_t)Lq, (int)hq, (int)hkv, std::min(p.ring, USP_MAX_RING_BLOCKS), true, !p.causal);
  f.copies.dq_stride = q_elems;
  f.copies.dkdv_stride = kv_elems;
  f.dkdv_copies = (int)(hq / hkv) / f.copies.cut.heads_per_wg * f.copies.cut.q_splits;
  f.kv_acc_bytes = up256(kv_elems * sizeof(float) * f.dkdv_copies);
  const size_t blocks = (size_t)p.ring * n_cols;
  size_t off = 0;
  const bool in_place = p.ulysses == 1;
  f.q_head = off; off += in_place ? 0 : qb;
  f.do_head = off; off += in_place ? 0 : qb;
  f.delta = off; off += up256((size_t)p.bs * hq * Lq * sizeof(float));
  f.k_head = off; off += in_place ? 0 : up256(f.kv_block_bytes * blocks);
  f.v_head = off; off += in_place ? 0 : up256(f.kv_block_bytes * blocks);
  f.dq_acc = off; off += up256(q_elems * sizeof(float) * f.copies.cut.k_splits);
  f.dk_acc = off; off += f.kv_acc_bytes * blocks;
  f.dv_acc = off; off += f.kv_acc_bytes * blocks;
  f.total = off;
  f.ds = off;
  // dS is kept only at head size 128: at 64 forming S and dP a second time costs less than moving 4 bytes per pair
  // (measured: 2.32 ms recomputed against 2.46 ms with dS kept on the Ulysses-8 rank of L = 32768)
  f.ds_bytes = bwd_keeps_ds(p.hs) ? up256(bwd_ds_bytes(p.bs, (int64_t)Lq, (int64_t)Lq, (int)hq, std::min(p.ring, USP_MAX_RING_BLOCKS))) : 0;
  f.total_with_ds = off + f.ds_bytes;
  return f;
}

}  // namespace

extern "C" size_t usp_attn_bwd_workspace_bytes(const usp_problem* p, int n_ranks) {
  if (usp_validate(p) != USP_OK || n_ranks < 1 || p->dtype != USP_BF16) return 0;
  const int cols = n_ranks == 1 ? 1 : p->ulysses;
  return plan_bwd(*p, cols).total;
}

extern "C" size_t usp_attn_bwd_workspace_bytes_with_ds(const usp_problem* p, int n_ranks) {
  if (usp_validate(p) != USP_OK || n_ranks < 1 || p->dtype != USP_BF16) return 0;
  const int cols = n_ranks == 1 ? 1 : p->ulysses;
  return plan_bwd(*p, cols).total_with_ds;
}

extern "C" int usp_attn_bwd(const usp_problem* p, const void* q, const void* k, const void* v, const void* o,
                            const float* lse, const void* d_o, void* dq, void* dk, void* dv, int rank_begin,
                            int rank_end, void* workspace, size_t workspace_bytes, void* stream_) {
  int st = usp_validate(p);
  if (st != USP_OK) return st;
  if (p->dtype != USP_BF16) return USP_ERR_DTYPE;
  if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return USP_ERR_NULL;
  const int U = p->ulysses, R = p->ring, N = U * R;
  if (rank_begin < 0 || rank_end > N || rank_begin >= rank_end) return USP_ERR_UNSUPPORTED;
  int c0, c1;
  column_range(*p, rank_begin, rank_end, &c0, &c1);
  const int n_cols = c1 - c0;
  BwdPlan f = plan_bwd(*p, n_cols);
  if (!workspace || workspace_bytes < f.total) return USP_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 255) return USP_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  char* ws = (char*)workspace;
  if (f.ds_bytes && workspace_bytes >= f.total_with_ds) f.copies.ds = ws + f.ds;   // room to keep dS between the two kernels
  const int64_t Lq = p->L / R;
  const int hq = p->hc / U, hkv = p->hk / U;
  const float scale = p->scale == 0.0f ? 1.0f / sqrtf((float)p->hs) : p->scale;
  const size_t q_elems = (size_t)p->bs * Lq * hq * p->hs, kv_elems = (size_t)p->bs * Lq * hkv * p->hs;
  auto slot = [&](int r, int u) { return (size_t)r * n_cols + (u - c0); };

  // Ulysses degree 1: the all-to-alls are the identity, a rank's Q / dO and every K/V block are shards as they stand
  const bool in_place = U == 1;
  const char* const k_blocks = in_place ? (const char*)k : ws + f.k_head;   // block slot 0 of K, of V
  const char* const v_blocks = in_place ? (const char*)v : ws + f.v_head;
  if (!in_place) {
    st = stage_kv_blocks(*p, k, v, ws + f.k_head, ws + f.v_head, f.kv_block_bytes, c0, c1, stream);
    if (st != USP_OK) return st;
  }

  // first contribution to a K/V block overwrites its accumulator, later ones add
  bool touched[USP_MAX_MERGE_PARTS] = {false};
  if ((size_t)R * n_cols > USP_MAX_MERGE_PARTS) return USP_ERR_UNSUPPORTED;

  for (int rank = rank_begin; rank < rank_end; ++rank) {
    const int r = rank / U, u = rank % U;
    const char* q_rank = (const char*)q + (size_t)rank * q_elems * dtype_size(p->dtype);      // used when in place
    const char* do_rank = (const char*)d_o + (size_t)rank * q_elems * dtype_size(p->dtype);
    if (!in_place) {   // Q and dO of this rank to head layout: one geometry, one launch
      const void* srcs[2] = {q, d_o};
      void* dsts[2] = {ws + f.q_head, ws + f.do_head};
      st = launch_layout_a2a_multi(*p, p->hc, USP_SEQ_TO_HEAD, 2, srcs, dsts, rank, rank + 1, rank, stream);
      if (st != USP_OK) return st;
      q_rank = ws + f.q_head;
      do_rank = ws + f.do_head;
    }
    // delta reads O (and dO) once: straight from the sequence-layout shards of the rank's Ulysses group, no copy of O
    float* delta = (float*)(ws + f.delta);
    {
      const SeqLayoutIO seq = {(int)(p->L / N), p->hc, u * hq};
      const size_t group_off = (size_t)r * U * p->bs * (p->L / N) * p->hc * p->hs * dtype_size(p->dtype);
      st = launch_bwd_delta((const char*)o + group_off, (const char*)d_o + group_off, delta, p->bs, Lq, hq, p->hs, stream, &seq);
      if (st != USP_OK) return st;
    }
    usp_posdesc qd;
    usp_local_positions(p, r, u, nullptr, &qd);
    const float* lse_rank = lse + (size_t)rank * p->bs * hq * Lq;
    // The ring loop of this rank, step i on block s = (r - i) mod R: up to USP_MAX_RING_BLOCKS steps per launch
    // pair (the dQ kernel keeps its accumulator in registers across them, the dK/dV kernel spreads them over
    // its grid).  dQ adds after the first launch of this rank; a block's dK/dV add after the first rank that
    // touched it.
    for (int i0 = 0; i0 < R; i0 += USP_MAX_RING_BLOCKS) {
      const int nb = R - i0 < USP_MAX_RING_BLOCKS ? R - i0 : USP_MAX_RING_BLOCKS;
      const void* kb[USP_MAX_RING_BLOCKS];
      const void* vb[USP_MAX_RING_BLOCKS];
      float* dkb[USP_MAX_RING_BLOCKS];
      float* dvb[USP_MAX_RING_BLOCKS];
      usp_posdesc kds[USP_MAX_RING_BLOCKS];
      int acc[USP_MAX_RING_BLOCKS];
      for (int j = 0; j < nb; ++j) {
        const int s = ((r - (i0 + j)) % R + R) % R;
        usp_local_positions(p, s, u, nullptr, &kds[j]);
        const size_t sl = slot(s, u);
        kb[j] = k_blocks + sl * f.kv_block_bytes;
        vb[j] = v_blocks + sl * f.kv_block_bytes;
        dkb[j] = (float*)(ws + f.dk_acc + sl * f.kv_acc_bytes);
        dvb[j] = (float*)(ws + f.dv_acc + sl * f.kv_acc_bytes);
        acc[j] = touched[sl] ? 1 : 0;
        touched[sl] = true;
      }
      st = launch_ring_attn_bwd(q_rank, kb, vb, kds, nb, do_rank, lse_rank, delta,
                                (float*)(ws + f.dq_acc), dkb, dvb, p->bs, Lq, Lq, hq, hkv, p->hs, scale,
                                p->causal ? 1 : 0, qd, i0 > 0 ? 1 : 0, acc, stream, &f.copies);
      if (st != USP_OK) return st;
    }
    // dQ of this rank: the copies summed, converted and written straight to the sequence-layout shards of its Ulysses
    // group (the reverse all-to-all rides on the conversion's stores)
    {
      const SeqLayoutIO seq = {(int)(p->L / N), p->hc, u * hq};
      const size_t group_off = (size_t)r * U * p->bs * (p->L / N) * p->hc * p->hs * dtype_size(p->dtype);
      st = launch_bwd_convert_seq((const float*)(ws + f.dq_acc), (char*)dq + group_off, nullptr, nullptr, q_elems, p->dtype,
                                  stream, f.copies.cut.k_splits, f.copies.dq_stride, 0, &seq, p->bs, Lq, hq, p->hs);
      if (st != USP_OK) return st;
    }
  }

  // dK, dV of every block the range touched: all ring rows of the columns whose ranks were run.  A range that
  // straddles ring rows without covering every column (say [U-1, U+1)) leaves columns between c0 and c1 unvisited:
  // their accumulators were never written, and their head slices of dk / dv stay as the caller left them.
  for (int r = 0; r < R; ++r)
    for (int u = c0; u < c1; ++u) {
      const int rank = r * U + u;
      const size_t sl = slot(r, u);
      if (!touched[sl]) continue;
      // the copies summed, converted and written straight to the block's sequence-layout shards
      const SeqLayoutIO seq = {(int)(p->L / N), p->hk, u * hkv};
      const size_t group_off = (size_t)r * U * p->bs * (p->L / N) * p->hk * p->hs * dtype_size(p->dtype);
      st = launch_bwd_convert_seq((const float*)(ws + f.dk_acc + sl * f.kv_acc_bytes), (char*)dk + group_off,
                                  (const float*)(ws + f.dv_acc + sl * f.kv_acc_bytes), (char*)dv + group_off, kv_elems,
                                  p->dtype, stream, f.dkdv_copies, f.copies.dkdv_stride, 0, &seq, p->bs, Lq, hkv, p->hs);
      if (st != USP_OK) return st;
    }
  return USP_OK;
}

extern "C" int usp_ring_attn_bwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                                 const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                                 const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks,
                                 int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                                 const usp_posdesc* qpos, int accumulate_dq, const int* accumulate_dkdv,
                                 void* stream) {
  if (!q || !k_blocks || !v_blocks || !d_o || !lse || !delta || !dq || !dk_blocks || !dv_blocks || !accumulate_dkdv)
    return USP_ERR_NULL;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return USP_ERR_UNSUPPORTED;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  usp_posdesc qd = {0, Lq, 0, 0};
  usp_posdesc kd[USP_MAX_RING_BLOCKS];
  int acc[USP_MAX_RING_BLOCKS];
  if (causal && (!qpos || !kpos_blocks)) return USP_ERR_NULL;
  if (causal && !desc_ok(qpos, Lq)) return USP_ERR_SHAPE;
  if (causal) qd = *qpos;
  for (int j = 0; j < n_blocks; ++j) {
    if (!k_blocks[j] || !v_blocks[j] || !dk_blocks[j] || !dv_blocks[j]) return USP_ERR_NULL;
    kd[j] = usp_posdesc{0, Lk, 0, 0};
    if (causal) {
      if (!desc_ok(&kpos_blocks[j], Lk)) return USP_ERR_SHAPE;
      kd[j] = kpos_blocks[j];
    }
    acc[j] = accumulate_dkdv[j] ? 1 : 0;
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  return launch_ring_attn_bwd(q, k_blocks, v_blocks, kd, n_blocks, d_o, lse, delta, dq, dk_blocks, dv_blocks, bs, Lq,
                              Lk, hq, hkv, hs, scale, causal ? 1 : 0, qd, accumulate_dq ? 1 : 0, acc,
                              (hipStream_t)stream);
}

namespace {

// Copies of the outputs that usp_ring_attn_bwd_ws keeps in its workspace: dq when its items are cut, every block's
// dk and dv when they have more than one writer per element.
struct RingBwdWs {
  BwdCopies copies;
  int dkdv_copies;
  size_t dq_bytes, kv_bytes_per_block, total;   // dq_bytes / kv_bytes_per_block are 0 where the output is written directly
  size_t ds_bytes, total_with_ds;               // room for dS behind the copies: used when the workspace reaches that far
};

RingBwdWs plan_ring_bwd_ws(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs, int n_blocks) {
  RingBwdWs w;
  w.copies.cut = plan_bwd_cut(bs, Lq, Lk, hq, hkv, n_blocks, true, false);
  w.copies.dq_stride = (size_t)bs * Lq * hq * hs;
  w.copies.dkdv_stride = (size_t)bs * Lk * hkv * hs;
  w.dkdv_copies = (hq / hkv) / w.copies.cut.heads_per_wg * w.copies.cut.q_splits;
  w.dq_bytes = w.copies.cut.k_splits > 1 ? up256(w.copies.dq_stride * sizeof(float) * w.copies.cut.k_splits) : 0;
  w.kv_bytes_per_block = w.dkdv_copies > 1 ? up256(w.copies.dkdv_stride * sizeof(float) * w.dkdv_copies) : 0;
  w.total = w.dq_bytes + 2 * w.kv_bytes_per_block * n_blocks;
  w.ds_bytes = bwd_keeps_ds(hs) ? up256(bwd_ds_bytes(bs, Lq, Lk, hq, n_blocks)) : 0;
  w.total_with_ds = w.total + w.ds_bytes;
  return w;
}

}  // namespace

extern "C" size_t usp_ring_attn_bwd_workspace_bytes(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                                                    int n_blocks) {
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1 || hq % hkv || (hs != 64 && hs != 128)) return 0;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return 0;
  return plan_ring_bwd_ws(bs, Lq, Lk, hq, hkv, hs, n_blocks).total;
}

extern "C" size_t usp_ring_attn_bwd_workspace_bytes_with_ds(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                                                            int n_blocks) {
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1 || hq % hkv || (hs != 64 && hs != 128)) return 0;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return 0;
  return plan_ring_bwd_ws(bs, Lq, Lk, hq, hkv, hs, n_blocks).total_with_ds;
}

extern "C" int usp_ring_attn_bwd_ws(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                                    const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                                    const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks,
                                    int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                                    const usp_posdesc* qpos, int accumulate_dq, const int* accumulate_dkdv,
                                    void* workspace, size_t workspace_bytes, void* stream_) {
  if (!q || !k_blocks || !v_blocks || !d_o || !lse || !delta || !dq || !dk_blocks || !dv_blocks || !accumulate_dkdv)
    return USP_ERR_NULL;
  if (n_blocks < 1 || n_blocks > USP_MAX_RING_BLOCKS) return USP_ERR_UNSUPPORTED;
  if (bs < 1 || Lq < 1 || Lk < 1 || hq < 1 || hkv < 1) return USP_ERR_SHAPE;
  if (hq % hkv) return USP_ERR_DEGREE;
  if (hs != 64 && hs != 128) return USP_ERR_UNSUPPORTED;
  if (!(scale >= 0.0f) || isinf(scale)) return USP_ERR_UNSUPPORTED;
  if (Lq >= (int64_t)1 << 31 || Lk >= (int64_t)1 << 31) return USP_ERR_UNSUPPORTED;
  RingBwdWs w = plan_ring_bwd_ws(bs, Lq, Lk, hq, hkv, hs, n_blocks);
  if (w.total > 0 && (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255))) return USP_ERR_WORKSPACE;
  if (w.ds_bytes && workspace && workspace_bytes >= w.total_with_ds && !((uintptr_t)workspace & 255))
    w.copies.ds = (char*)workspace + w.total;   // room to keep dS between the two kernels
  usp_posdesc qd = {0, Lq, 0, 0};
  usp_posdesc kd[USP_MAX_RING_BLOCKS];
  if (causal && (!qpos || !kpos_blocks)) return USP_ERR_NULL;
  if (causal && !desc_ok(qpos, Lq)) return USP_ERR_SHAPE;
  if (causal) qd = *qpos;
  hipStream_t stream = (hipStream_t)stream_;
  char* ws = (char*)workspace;
  // where the kernels write: the copies in the workspace (always overwritten there), or the outputs themselves
  float* dq_dst = w.dq_bytes ? (float*)ws : dq;
  float* dk_dst[USP_MAX_RING_BLOCKS];
  float* dv_dst[USP_MAX_RING_BLOCKS];
  int acc[USP_MAX_RING_BLOCKS];
  for (int j = 0; j < n_blocks; ++j) {
    if (!k_blocks[j] || !v_blocks[j] || !dk_blocks[j] || !dv_blocks[j]) return USP_ERR_NULL;
    kd[j] = usp_posdesc{0, Lk, 0, 0};
    if (causal) {
      if (!desc_ok(&kpos_blocks[j], Lk)) return USP_ERR_SHAPE;
      kd[j] = kpos_blocks[j];
    }
    if (w.kv_bytes_per_block) {
      dk_dst[j] = (float*)(ws + w.dq_bytes + (size_t)(2 * j) * w.kv_bytes_per_block);
      dv_dst[j] = (float*)(ws + w.dq_bytes + (size_t)(2 * j + 1) * w.kv_bytes_per_block);
      acc[j] = 0;
    } else {
      dk_dst[j] = dk_blocks[j];
      dv_dst[j] = dv_blocks[j];
      acc[j] = accumulate_dkdv[j] ? 1 : 0;
    }
  }
  if (scale == 0.0f) scale = 1.0f / sqrtf((float)hs);
  int st = launch_ring_attn_bwd(q, k_blocks, v_blocks, kd, n_blocks, d_o, lse, delta, dq_dst, dk_dst, dv_dst, bs, Lq, Lk,
                                hq, hkv, hs, scale, causal ? 1 : 0, qd, w.dq_bytes ? 0 : (accumulate_dq ? 1 : 0), acc,
                                stream, &w.copies);
  if (st != USP_OK) return st;
  if (w.dq_bytes) {
    st = launch_bwd_convert(dq_dst, dq, w.copies.dq_stride, USP_FP32, stream, w.copies.cut.k_splits, w.copies.dq_stride,
                            accumulate_dq ? 1 : 0);
    if (st != USP_OK) return st;
  }
  if (w.kv_bytes_per_block)
    for (int j = 0; j < n_blocks; ++j) {
      st = launch_bwd_convert(dk_dst[j], dk_blocks[j], w.copies.dkdv_stride, USP_FP32, stream, w.dkdv_copies,
                              w.copies.dkdv_stride, accumulate_dkdv[j] ? 1 : 0);
      if (st != USP_OK) return st;
      st = launch_bwd_convert(dv_dst[j], dv_blocks[j], w.copies.dkdv_stride, USP_FP32, stream, w.dkdv_copies,
                              w.copies.dkdv_stride, accumulate_dkdv[j] ? 1 : 0);
      if (st != USP_OK) return st;
    }
  return USP_OK;
}
