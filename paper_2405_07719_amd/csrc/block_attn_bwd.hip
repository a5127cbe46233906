// Backward of one ring step of blockwise attention (textbook gradient of Eq. 1, Sec. 2, restricted to one
// K/V block; the paper only says that the backward all-to-alls swap their scatter/gather roles, Sec. 3).
//
// With the FINAL log-sum-exp L_i of a query row (over all keys of all blocks) and D_i = sum_e dO_ie O_ie:
//   P_ij = exp(scale q_i.k_j - L_i),  dV_j = sum_i P_ij dO_i,  dS_ij = P_ij (dO_i.v_j - D_i),
//   dQ_i = scale sum_j dS_ij k_j,     dK_j = scale sum_i dS_ij q_i.
// P and dS are exact per element, so the contributions of different K/V blocks simply add.
//
// Two kernels, both on v_mfma_f32_32x32x16_bf16 with fp32 accumulation:
//   dq_kernel    a workgroup owns 256 query rows, walks the visible key tiles:  S^T = K Q^T, dP^T = V dO^T
//                (lane = query, so L_i and D_i are per-lane scalars), dQ^T += K^T dS^T.  Deterministic.
//   dkdv_kernel  a workgroup owns 256 keys of one KV head and walks the visible query tiles of one query
//                head, or of all query heads of the group when the grid is large enough without splitting them:
//                S = Q K^T, dP = dO V^T (lane = key; L_i and D_i enter through one extra MFMA k-step),
//                dV^T += dO^T P, dK^T += Q^T dS; split heads meet through fp32 atomic adds.
// Both take up to USP_MAX_RING_BLOCKS K/V blocks per launch (the ring loop of one rank).
// In both, the accumulator layout of the first product is the B-operand layout of the second, and the
// transposed A operands come from LDS transpose reads of the same tile copy: a row stride of 2*hs + 48 bytes is
// free of bank conflicts for the 16 B row reads and for the transpose reads alike.
// Outputs are fp32 accumulators (overwrite or add), so ring steps and ranks can be summed before the
// final conversion to the problem dtype.
#include <algorithm>
#include <numeric>

#include "attn_device.h"
#include "usp_internal.h"

namespace usp {
namespace {

using namespace dev;

constexpr int kMaxBlocks = USP_MAX_RING_BLOCKS;

// One launch covers the n_blocks K/V blocks of a rank's ring loop (n_blocks = 1: a single ring step): the dQ
// kernel walks them one after the other with its accumulator in registers, the dK/dV kernel spreads them over
// the grid (each block has its own output accumulators).
struct BwdArgs {
  const void* q;
  const void* k[kMaxBlocks];
  const void* v[kMaxBlocks];
  const void* d_o;
  const float* lse;     // [bs,hq,Lq]  final LSE (natural log)
  const float* delta;   // [bs,hq,Lq]  D_i
  float* dq;            // [bs,Lq,hq,hs]  fp32
  float* dk[kMaxBlocks];   // [bs,Lk,hkv,hs] fp32 per block
  float* dv[kMaxBlocks];
  int bs, hq, hkv, g;
  int Lq, Lk;
  int n_tiles;          // query tiles (dq) or key tiles per block (dkdv)
  int n_blocks;
  int causal;
  int accumulate;       // dq: 0 overwrite, 1 add
  int heads_per_wg;     // dkdv: query heads of a KV group walked by one workgroup (g: plain stores; else atomics)
  int acc_dkdv[kMaxBlocks];   // dkdv with heads_per_wg == g: 0 overwrite the block's dK/dV, 1 add to them
  float scale, scale_log2;
  PosDesc32 qpos;
  PosDesc32 kpos[kMaxBlocks];
  // the workgroups of both kernels are persistent and draw their work items (attn_device.h); set per launch
  int ticket_slot, n_items, n_queues;
  // Short sequences (few, long work items): the dQ kernel's items are cut into k_splits slices of their visible key
  // tiles, the dK/dV kernel's into q_splits slices of their visible query tiles.  Slice s of the dQ kernel writes the
  // s-th copy of dq, dq_part_stride elements further on; part (head split x q_splits + query slice) of the dK/dV
  // kernel writes that copy of the block's dk and dv, dkdv_part_stride elements further on (no atomics then); the
  // caller adds the copies up (launch_bwd_convert).  1 and 0 = not cut, one copy.
  int k_splits, q_splits;
  size_t dq_part_stride, dkdv_part_stride;
  // dS kept between the two kernels (null: each kernel forms its own).  The dK/dV kernel, which runs first then,
  // writes every 32 x 32 block of dS it forms, unscaled, as bf16 [query half][key][16 queries] (2 KiB), block (head, K/V block, key
  // tile kt, query tile qt) at index ((((b hq + h) n_blocks + blk) ds_qt8 + qt / 8) ds_kt + kt) 8 + qt % 8: what
  // a workgroup of the dQ kernel (256 queries: qt / 8) reads, key tile after key tile, is one contiguous stream.
  // The dQ kernel reads the blocks that hold a visible pair (all of those have been written) and is left with
  // one product, dQ^T += K^T dS^T.
  void* ds;
  int ds_kt, ds_qt8;    // per K/V block: blocks along the keys (a multiple of 8: whole 256-key tiles), 256-query tiles
};

// The scalar arguments as one work item of the dQ kernel sees them (read anew for every item, see the kernel).
struct DqItemArgs {
  const void* q;
  const void* d_o;
  const float* lse;
  const float* delta;
  float* dq;
  int bs, hq, hkv, g;
  int Lq, Lk;
  int n_tiles, n_blocks, causal, accumulate;
  float scale, scale_log2;
  PosDesc32 qpos;
};

// ... and of the dK/dV kernel.
struct DkdvItemArgs {
  const void* q;
  const void* d_o;
  const float* lse;
  const float* delta;
  int bs, hq, hkv, g;
  int Lq, Lk;
  int n_tiles, causal, heads_per_wg;
  float scale, scale_log2;
  PosDesc32 qpos;
};

constexpr float kLog2e = 1.4426950408889634f;
// A stored 32 x 32 block of dS is two halves of 1 KiB, [query half][key][16 queries]: every 16-byte store
// instruction of the writer fills whole 128-byte lines.  In the reader's LDS the second half sits 1152 bytes after
// the first (an odd multiple of 128: the two 16-lane groups of a transpose read then hit different banks).
constexpr int kDsHalfLds = 1152, kDsBlockLds = kDsHalfLds + 1024;
// Cache policy of the dS stores: non-temporal (bit 1 of the buffer instructions' policy operand).  Nothing reads the
// blocks before the next kernel, and kept as ordinary dirty lines they push the Q / dO rows out of the L2s.  (With
// whole lines per store instruction this is 2-3 % faster over the kernel pair than the default policy; when a
// store instruction filled half lines it was 10 % slower.)
constexpr int kDsStoreAux = 2;

// transpose-read address of this lane inside a [rows][VSTR] tile: see the forward kernel
template <int VSTR>
__device__ inline int tr_lane_offset(int lane) {
  const int hl = lane >> 5, grp = lane >> 4, j16 = lane & 15;
  return (4 * hl + (j16 >> 2)) * VSTR + (16 * (grp & 1) + 4 * (j16 & 3)) * 2;
}

template <int VSTR>
__device__ inline bf16x8 tr_read(const char* p0) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * VSTR));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ inline void zero16(f32x16& x) {
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.f;
}

// 16 fp32 values of a 32x32 accumulator block -> two bf16 B-operand fragments (k-steps of 16)
__device__ inline void pack_b_operand(const float (&x)[16], bf16x8& lo, bf16x8& hi) {
  u32x4 a, b;
#pragma unroll
  for (int pr = 0; pr < 4; ++pr) {
    a[pr] = pack_bf16(x[2 * pr], x[2 * pr + 1]);
    b[pr] = pack_bf16(x[8 + 2 * pr], x[8 + 2 * pr + 1]);
  }
  lo = __builtin_bit_cast(bf16x8, a);
  hi = __builtin_bit_cast(bf16x8, b);
}

// -------------------------------------------------------------------------------------------------
// D_i = sum_e dO_ie * O_ie   (rows of [bs,L,h,hs] tensors -> [bs,h,L] fp32)
// -------------------------------------------------------------------------------------------------
// seq_n > 0: o and d_o are not dense [bs, L, h, hs] tensors but the sequence-layout shards of the rank's Ulysses group
// ([U][bs][seq_n][seq_heads][hs], the rank's h heads from seq_head0 on): row i of the rank lies in shard i / seq_n.
template <int HS>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const __bf16* o, const __bf16* d_o, float* delta, int bs,
                                                        int L, int h, int seq_n, int seq_heads, int seq_head0) {
  constexpr int TPR = HS / 8;   // lanes per row, 8 elements each
  const int64_t rows = (int64_t)bs * L * h;
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) / TPR;
  const int part = threadIdx.x % TPR;
  float acc = 0.f;
  if (row < rows) {
    int64_t at = row;   // the row's place in o and d_o, in rows of HS elements
    if (seq_n) {
      const int64_t hh = row % h, i = (row / h) % L, b = row / ((int64_t)h * L);
      const int64_t shard = i / seq_n, sr = i - shard * seq_n;
      at = ((shard * bs + b) * seq_n + sr) * seq_heads + seq_head0 + hh;
    }
    const bf16x8 a = *(const bf16x8*)(o + at * HS + part * 8);
    const bf16x8 b = *(const bf16x8*)(d_o + at * HS + part * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
  }
#pragma unroll
  for (int m = TPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (row < rows && part == 0) {
    const int64_t hh = row % h, i = (row / h) % L, b = row / ((int64_t)h * L);
    delta[(b * h + hh) * L + i] = acc;
  }
}

// -------------------------------------------------------------------------------------------------
// dQ
// -------------------------------------------------------------------------------------------------
template <int HS>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void bwd_dq_kernel(const BwdArgs) {
  constexpr int NT = 512, BM = 256, KT = 32;
  constexpr int KSTEPS = HS / 16, DB = HS / 32;
  constexpr int USTR = HS * 2 + 48;                 // conflict-free for 16 B row reads and for transpose reads
  constexpr int CPR = HS / 8;                       // 16 B chunks per row
  constexpr int STAGE = 2 * KT * USTR;              // K, V
  static_assert(KT * CPR <= NT, "one chunk per thread and tensor");
  __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];

  // Persistent workgroups, one per CU, that draw their work items as the forward kernel's do (same item order:
  // KV group fastest, then head within group, then query tile, heavy first; the next item is asked for at the start
  // of the epilogue and the answer read after the stores).
  __shared__ int next_item[2];
  __shared__ unsigned empty_queues;
  int turn = 0;
  if (threadIdx.x == 0) {
    auto ap0 = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    // the first item is given, not drawn
    next_item[0] = ItemQueues{ap0->ticket_slot, ap0->n_items, (int)gridDim.x, ap0->n_queues}.first_item(blockIdx.x);
    empty_queues = 0;
  }
  for (;;) {
    // arguments and lane constants are read / derived anew for every item, so that nothing derived from them is
    // carried in registers across the item loop
    auto ap = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
    const ItemQueues queues = {ap->ticket_slot, ap->n_items, (int)gridDim.x, ap->n_queues};
    __syncthreads();   // the previous item is done with LDS, and next_item[turn] has been written
    int w = __builtin_amdgcn_readfirstlane(next_item[turn]);
    turn ^= 1;
    if (w >= queues.n_items) {
      if (threadIdx.x == 0) queues.leave();
      break;
    }
    DqItemArgs a;
    a.q = ap->q; a.d_o = ap->d_o; a.lse = ap->lse; a.delta = ap->delta; a.dq = ap->dq;
    a.bs = ap->bs; a.hq = ap->hq; a.hkv = ap->hkv; a.g = ap->g;
    a.Lq = ap->Lq; a.Lk = ap->Lk;
    a.n_tiles = ap->n_tiles; a.n_blocks = ap->n_blocks; a.causal = ap->causal; a.accumulate = ap->accumulate;
    a.scale = ap->scale; a.scale_log2 = ap->scale_log2;
    a.qpos = PosDesc32{ap->qpos.start0, ap->qpos.len0, ap->qpos.start1, ap->qpos.len1};
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keep what derives from it in scalar registers
    const int l32 = lane & 31, hl = lane >> 5;
    const int n_groups = a.bs * a.hkv;
    const int group = w % n_groups; w /= n_groups;
    const int hg = w % a.g; w /= a.g;
    const int k_splits = ap->k_splits;
    const int kslice = w % k_splits;             // this item's slice of the visible key tiles of every block
    const int t = w / k_splits;
    const int qtile = a.causal ? a.n_tiles - 1 - t : t;
    const int b = group / a.hkv, kvh = group % a.hkv;
    const int h = kvh * a.g + hg;
    const int tile_row0 = qtile * BM, tile_row1 = min(a.Lq, tile_row0 + BM);
    const int wave_row0 = tile_row0 + wave * 32;
    const int qrow = wave_row0 + l32;
    const int rr = min(qrow, a.Lq - 1);
    const int qp = a.causal ? pos_of(a.qpos, rr) : 0;

    const size_t kv_head_off = ((size_t)b * a.Lk * a.hkv + kvh) * HS * 2;   // bytes
    const char* kg = nullptr;   // per block, set at the top of the block loop
    const char* vg = nullptr;
    const uint32_t row_bytes = (uint32_t)a.hkv * HS * 2;

    bf16x8 qf[KSTEPS], dof[KSTEPS];
    {
      const size_t off = (((size_t)b * a.Lq + rr) * a.hq + h) * HS + 8 * hl;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        qf[ks] = *(const bf16x8*)((const __bf16*)a.q + off + 16 * ks);
        dof[ks] = *(const bf16x8*)((const __bf16*)a.d_o + off + 16 * ks);
      }
    }
    const size_t stat = ((size_t)b * a.hq + h) * a.Lq + rr;
    const float lse = a.lse[stat];
    float dlt = a.delta[stat];
    float l2 = (lse == -INFINITY) ? INFINITY : lse * kLog2e;   // a row that saw nothing: P = 0
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      settle(qf[ks]);
      settle(dof[ks]);
    }
    settle(l2);
    settle(dlt);

    f32x16 dq[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) zero16(dq[db]);

    PosDesc32 kpos = {0, 0, 0, 0};
    TileRanges tr = {0, 0, 0, 0};
    int na = 0, nt = 0;
    auto tile_of = [&](int it) { return it < na ? tr.a0 + it : tr.b0 + (it - na); };
    const bool wave_live = wave_row0 < a.Lq;
    const int wave_qmin = (a.causal && wave_live) ? pos_min(a.qpos, wave_row0, min(a.Lq, wave_row0 + 32)) : 0;

    // staging: one 16 B chunk of K and of V per thread and tile; the tile base is wave-uniform, the per-thread
    // byte offset constant, rows past the last key clamped by a min on the offset
    const int st_row = tid / CPR, st_col = tid % CPR;
    const bool stager = st_row < KT;
    const uint32_t st_off = (uint32_t)st_row * row_bytes + st_col * 16;
    u32x4 kreg, vreg;
    auto fetch = [&](int it) {
      if (stager) {
        const int key0 = tile_of(it) * KT;
        const uint32_t lim = (uint32_t)min(a.Lk - 1 - key0, KT - 1) * row_bytes + st_col * 16;
        const uint32_t off = min(st_off, lim);
        kreg = *(const u32x4*)(kg + (size_t)key0 * row_bytes + off);
        vreg = *(const u32x4*)(vg + (size_t)key0 * row_bytes + off);
      }
    };
    auto stash = [&](int buf) {
      if (stager) {
        char* base = lds + buf * STAGE;
        *(u32x4*)(base + st_row * USTR + st_col * 16) = kreg;
        *(u32x4*)(base + KT * USTR + st_row * USTR + st_col * 16) = vreg;
      }
    };
    const int tr_off = tr_lane_offset<USTR>(lane);
    const int row_off = l32 * USTR + hl * 16;

    for (int blk = 0; blk < a.n_blocks; ++blk) {
    kpos = PosDesc32{ap->kpos[blk].start0, ap->kpos[blk].len0, ap->kpos[blk].start1, ap->kpos[blk].len1};
    tr = visible_key_tiles<KT>(a.causal, a.qpos, kpos, a.Lk, tile_row0, tile_row1);
    na = tr.a1 - tr.a0;
    nt = na + (tr.b1 - tr.b0);
    const int it0 = (int)((int64_t)nt * kslice / k_splits), it1 = (int)((int64_t)nt * (kslice + 1) / k_splits);
    if (it1 == it0) continue;                // workgroup-uniform
    // Tiles this wave need not mask: full tiles that lie wholly in one ascending run of the key positions and whose
    // last key none of the wave's rows precedes.  In walk order they are [0, free_a) and [free_b0, free_b1), worked
    // out here once per block; the decision per tile is then two comparisons.
    int free_a, free_b0, free_b1;
    {
      const int full = a.Lk / KT;
      int fa = full, tb0 = 0, tb1 = 0;
      if (a.causal && wave_live) {
        int64_t c0 = (int64_t)wave_qmin - kpos.start0 + 1; c0 = c0 < 0 ? 0 : (c0 > kpos.len0 ? kpos.len0 : c0);
        int64_t c1 = (int64_t)wave_qmin - kpos.start1 + 1; c1 = c1 < 0 ? 0 : (c1 > kpos.len1 ? kpos.len1 : c1);
        fa = (int)(c0 / KT);
        tb0 = (int)(((int64_t)kpos.len0 + KT - 1) / KT);
        tb1 = (int)(((int64_t)kpos.len0 + c1) / KT);
      }
      free_a = min(min(fa, full), na);
      free_b0 = na + max(tb0, tr.b0) - tr.b0;
      free_b1 = na + min(min(tb1, full), tr.b1) - tr.b0;
    }
    kg = (const char*)ap->k[blk] + kv_head_off;
    vg = (const char*)ap->v[blk] + kv_head_off;
    fetch(it0);
    stash(it0 & 1);                          // the previous block's last step ended on a barrier
    __syncthreads();
    for (int it = it0; it < it1; ++it) {
      const bool more = it + 1 < it1;
      if (more) fetch(it + 1);
      __builtin_amdgcn_sched_barrier(0);     // keep the loads above the compute (the scheduler would sink them)
      const char* k_s = lds + (it & 1) * STAGE;
      const char* v_s = k_s + KT * USTR;
      const int key0 = tile_of(it) * KT;

      // S^T = K Q^T and dP^T = V dO^T   (rows = keys, cols = queries)
      f32x16 s, dp;
      zero16(s);
      zero16(dp);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const bf16x8 kf = *(const bf16x8*)(k_s + row_off + ks * 32);
        const bf16x8 vf = *(const bf16x8*)(v_s + row_off + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[ks], dp, 0, 0, 0);
      }

      const bool need_mask = !(it < free_a || (it >= free_b0 && it < free_b1));
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], a.scale_log2, -l2));
      if (need_mask) {     // wave-uniform and rare: tiles on the causal boundary or the ragged tail
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = key0 + 8 * (i >> 2) + 4 * hl + (i & 3);
          const bool vis = key < a.Lk && (!a.causal || pos_of(kpos, key) <= qp);
          s[i] = vis ? s[i] : 0.f;
        }
      }
      float ds[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) ds[i] = s[i] * (dp[i] - dlt);
      bf16x8 dsf[2];
      pack_b_operand(ds, dsf[0], dsf[1]);

      // dQ^T += K^T dS^T   (rows = head dims, cols = queries, k = keys)
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 kt = tr_read<USTR>(k_s + tr_off + (16 * st) * USTR + db * 64);
          dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, dsf[st], dq[db], 0, 0, 0);
        }
      if (more) stash((it + 1) & 1);
      __syncthreads();
    }
    }   // blocks

    unsigned own_ticket = kNoDraw;
    if (threadIdx.x == 0) own_ticket = queues.begin(empty_queues);
    if (qrow < a.Lq) {
      float* dst = a.dq + (size_t)kslice * ap->dq_part_stride + (((size_t)b * a.Lq + qrow) * a.hq + h) * HS + 4 * hl;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          f32x4 v4 = {dq[db][4 * j] * a.scale, dq[db][4 * j + 1] * a.scale, dq[db][4 * j + 2] * a.scale,
                      dq[db][4 * j + 3] * a.scale};
          f32x4* d = (f32x4*)(dst + db * 32 + j * 8);
          if (a.accumulate) v4 += *d;
          *d = v4;
        }
    }
    if (threadIdx.x == 0) {
      unsigned empty = empty_queues;
      next_item[turn] = queues.finish(own_ticket, empty);
      empty_queues = empty;
    }
  }   // next work item
}

// -------------------------------------------------------------------------------------------------
// dQ from a stored dS: what is left of the dQ kernel when the dK/dV kernel has written its dS blocks
// (BwdArgs::ds).  One product, dQ^T += K^T dS^T, and the kernel is bound by reading dS: 2 bytes per visible
// (query, key) pair.  Same work items, slices and epilogue as bwd_dq_kernel.  A step covers KT keys (64 or
// 128): the K rows staged by the workgroup (double buffered), and per wave KT / 32 blocks of dS (2 KiB: its 32
// queries x 32 keys each) that the wave copies as they are into its own part of LDS and reads back through
// transpose reads, which yields the B operand (lane = query, k = keys in the order of the K^T fragments).  A
// wave reads a step's blocks only when one of their (query, key) pairs is visible: the dK/dV kernel has written
// them all then (they lie in one of its 256-key tiles, which has a visible pair with this query tile); the
// others would be all zero, and may never have been written.
// -------------------------------------------------------------------------------------------------
template <int HS, int KT>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void bwd_dq_ds_kernel(const BwdArgs) {
  constexpr int NT = 512, BM = 256;
  constexpr int NB = KT / 32;                       // dS blocks per wave and step
  constexpr int DB = HS / 32;
  constexpr int USTR = HS * 2 + 48;
  constexpr int CPR = HS / 8;
  constexpr int CPT = KT * CPR / NT;                // 16 B chunks of K per thread and step
  constexpr int STAGE = KT * USTR;
  static_assert(KT * CPR % NT == 0, "whole chunks per thread");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* const lds = smem;                           // [2][STAGE]  K
  char* const ds_all = smem + 2 * STAGE;            // [8 waves][NB blocks] of kDsBlockLds bytes

  __shared__ int next_item[2];
  __shared__ unsigned empty_queues;
  int turn = 0;
  if (threadIdx.x == 0) {
    auto ap0 = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    next_item[0] = ItemQueues{ap0->ticket_slot, ap0->n_items, (int)gridDim.x, ap0->n_queues}.first_item(blockIdx.x);
    empty_queues = 0;
  }
  for (;;) {
    auto ap = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
    const ItemQueues queues = {ap->ticket_slot, ap->n_items, (int)gridDim.x, ap->n_queues};
    __syncthreads();   // the previous item is done with LDS, and next_item[turn] has been written
    int w = __builtin_amdgcn_readfirstlane(next_item[turn]);
    turn ^= 1;
    if (w >= queues.n_items) {
      if (threadIdx.x == 0) queues.leave();
      break;
    }
    const int bs = ap->bs, hq = ap->hq, hkv = ap->hkv, g = ap->g, Lq = ap->Lq, Lk = ap->Lk;
    const int causal = ap->causal, n_blocks = ap->n_blocks;
    const PosDesc32 qpos = {ap->qpos.start0, ap->qpos.len0, ap->qpos.start1, ap->qpos.len1};
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hl = lane >> 5;
    const int n_groups = bs * hkv;
    const int group = w % n_groups; w /= n_groups;
    const int hg = w % g; w /= g;
    const int k_splits = ap->k_splits;
    const int kslice = w % k_splits;
    const int t = w / k_splits;
    const int qtile = causal ? ap->n_tiles - 1 - t : t;
    const int b = group / hkv, kvh = group % hkv;
    const int h = kvh * g + hg;
    const int tile_row0 = qtile * BM, tile_row1 = min(Lq, tile_row0 + BM);
    const int wave_row0 = tile_row0 + wave * 32;
    const int qrow = wave_row0 + l32;
    const bool wave_live = wave_row0 < Lq;
    const int wave_qmax = (causal && wave_live) ? pos_max(qpos, wave_row0, min(Lq, wave_row0 + 32)) : 0;

    const size_t kv_head_off = ((size_t)b * Lk * hkv + kvh) * HS * 2;   // bytes
    const uint32_t row_bytes = (uint32_t)hkv * HS * 2;
    const char* kg = nullptr;      // per block
    const char* dsg = nullptr;     // per block: this wave's column of dS blocks (query tile qtile * 8 + wave)
    constexpr size_t ds_kt_stride = 8 * 2048;   // bytes from one key tile of 32 to the next: the workgroup's 8 blocks

    f32x16 dq[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) zero16(dq[db]);

    PosDesc32 kpos = {0, 0, 0, 0};
    TileRanges tr = {0, 0, 0, 0};
    int na = 0;
    auto tile_of = [&](int it) { return it < na ? tr.a0 + it : tr.b0 + (it - na); };
    // does this wave's query tile see a key of the step's KT?
    auto sees = [&](int it) {
      if (!wave_live) return false;
      if (!causal) return true;
      const int key0 = tile_of(it) * KT;
      return pos_min(kpos, key0, min(Lk, key0 + KT)) <= wave_qmax;
    };

    const int st_row = tid / CPR, st_col = tid % CPR;      // first chunk; chunk c is (NT / CPR) rows further down
    const uint32_t st_off = (uint32_t)st_row * row_bytes + st_col * 16;
    u32x4 kreg[CPT], dreg[2 * NB];
    auto fetch = [&](int it, bool seen) {
      const int key0 = tile_of(it) * KT;
      const uint32_t last = (uint32_t)min(Lk - 1 - key0, KT - 1) * row_bytes + st_col * 16;   // rows past the last key: clamped
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        kreg[c] = *(const u32x4*)(kg + (size_t)key0 * row_bytes + min(st_off + c * (NT / CPR) * row_bytes, last));
      if (seen) {
        const char* blk0 = dsg + (size_t)(NB * tile_of(it)) * ds_kt_stride + lane * 16;
#pragma unroll
        for (int j = 0; j < 2 * NB; ++j)   // read once: streamed past the caches
          dreg[j] = __builtin_nontemporal_load((const u32x4*)(blk0 + (j >> 1) * ds_kt_stride + (j & 1) * 1024));
      }
    };
    char* const ds_s = ds_all + wave * (NB * kDsBlockLds);
    auto stash = [&](int buf, bool seen) {
      char* base = lds + buf * STAGE;
#pragma unroll
      for (int c = 0; c < CPT; ++c) *(u32x4*)(base + (st_row + c * (NT / CPR)) * USTR + st_col * 16) = kreg[c];
      if (seen) {
#pragma unroll
        for (int j = 0; j < 2 * NB; ++j) *(u32x4*)(ds_s + (j >> 1) * kDsBlockLds + (j & 1) * kDsHalfLds + lane * 16) = dreg[j];
      }
    };
    const int tr_off = tr_lane_offset<USTR>(lane);
    // transpose-read address inside a block: 32-byte rows of one half, the halves kDsHalfLds apart
    const int tr_off_ds = (4 * (lane >> 5) + ((lane & 15) >> 2)) * 32 + ((lane >> 4) & 1) * kDsHalfLds + (lane & 3) * 8;

    for (int blk = 0; blk < n_blocks; ++blk) {
    kpos = PosDesc32{ap->kpos[blk].start0, ap->kpos[blk].len0, ap->kpos[blk].start1, ap->kpos[blk].len1};
    tr = visible_key_tiles<KT>(causal, qpos, kpos, Lk, tile_row0, tile_row1);
    na = tr.a1 - tr.a0;
    const int nt = na + (tr.b1 - tr.b0);
    const int it0 = (int)((int64_t)nt * kslice / k_splits), it1 = (int)((int64_t)nt * (kslice + 1) / k_splits);
    if (it1 == it0) continue;                // workgroup-uniform
    kg = (const char*)ap->k[blk] + kv_head_off;
    dsg = (const char*)ap->ds + (((((size_t)b * hq + h) * n_blocks + blk) * ap->ds_qt8 + qtile) * ap->ds_kt * 8 + wave) * 2048;
    bool seen = sees(it0);
    fetch(it0, seen);
    stash(it0 & 1, seen);                    // the previous block's last step ended on a barrier
    __syncthreads();
    for (int it = it0; it < it1; ++it) {
      const bool more = it + 1 < it1;
      const bool seen_next = more && sees(it + 1);
      bf16x8 dsf[2 * NB];
      if (seen) {
#pragma unroll
        for (int st = 0; st < 2 * NB; ++st) dsf[st] = tr_read<32>(ds_s + (st >> 1) * kDsBlockLds + (16 * (st & 1)) * 32 + tr_off_ds);
      }
      if (more) fetch(it + 1, seen_next);
      __builtin_amdgcn_sched_barrier(0);     // keep the loads above the compute
      const char* k_s = lds + (it & 1) * STAGE;
      if (seen) {
        // dQ^T += K^T dS^T   (rows = head dims, cols = queries, k = keys)
#pragma unroll
        for (int st = 0; st < 2 * NB; ++st)
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const bf16x8 kt = tr_read<USTR>(k_s + tr_off + (16 * st) * USTR + db * 64);
            dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, dsf[st], dq[db], 0, 0, 0);
          }
      }
      if (more) stash((it + 1) & 1, seen_next);
      seen = seen_next;
      __syncthreads();
    }
    }   // blocks

    unsigned own_ticket = kNoDraw;
    if (threadIdx.x == 0) own_ticket = queues.begin(empty_queues);
    if (qrow < Lq) {
      const float scale = ap->scale;
      const int accumulate = ap->accumulate;
      float* dst = ap->dq + (size_t)kslice * ap->dq_part_stride + (((size_t)b * Lq + qrow) * hq + h) * HS + 4 * hl;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          f32x4 v4 = {dq[db][4 * j] * scale, dq[db][4 * j + 1] * scale, dq[db][4 * j + 2] * scale,
                      dq[db][4 * j + 3] * scale};
          f32x4* d = (f32x4*)(dst + db * 32 + j * 8);
          if (accumulate) v4 += *d;
          *d = v4;
        }
    }
    if (threadIdx.x == 0) {
      unsigned empty = empty_queues;
      next_item[turn] = queues.finish(own_ticket, empty);
      empty_queues = empty;
    }
  }   // next work item
}

// -------------------------------------------------------------------------------------------------
// dK, dV.  A workgroup owns 256 keys of one KV head (eight waves of 32 keys) and ONE query head of its
// group, and walks the visible query tiles of 32 rows, double buffered in LDS.  The query heads of a
// group (and nothing else) meet in the fp32 outputs through atomic adds: at most hq/hkv addends per
// element, the only non-deterministic rounding of the backward.
// -------------------------------------------------------------------------------------------------
template <int HS, bool WRITE_DS>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void bwd_dkdv_kernel(const BwdArgs) {
  constexpr int NT = 512, BN = 256, QT = 32;
  constexpr int KSTEPS = HS / 16, DB = HS / 32;
  constexpr int USTR = HS * 2 + 48;        // one row stride that is conflict-free for 16 B row reads AND transpose reads
  constexpr int CPR = HS / 8;
  constexpr int STAGE = 2 * QT * USTR;     // Q, dO (each row carries its statistic in the padding, see below)
  constexpr int XOFF = HS * 2;             // byte offset, inside a row, of the extra k-step that holds the statistic
  static_assert(QT * CPR <= NT, "one chunk per thread and tensor");
  static_assert(XOFF + 32 <= USTR, "the extra k-step lives in the row padding");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* const v_s = smem;                  // [BN][USTR]: the workgroup's V rows, resident for the whole kernel
  char* const lds = smem + BN * USTR;      // [2][STAGE]

  // the upper 16 bytes of the A rows' extra k-step (see stash below) are zeroed once: nothing else writes them
  if (threadIdx.x < 4 * QT)
    *(u32x4*)(lds + (threadIdx.x / QT) * (QT * USTR) + (threadIdx.x % QT) * USTR + XOFF + 16) = u32x4{0, 0, 0, 0};

  // Persistent workgroups, one per CU, that draw their work items as the forward kernel's do.  Item order: KV
  // group fastest, then the head split, then the key tile (ascending: keys seen by the most queries first), then
  // the K/V block of the ring loop.
  __shared__ int next_item[2];
  __shared__ unsigned empty_queues;
  int turn = 0;
  if (threadIdx.x == 0) {
    auto ap0 = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    // the first item is given, not drawn
    next_item[0] = ItemQueues{ap0->ticket_slot, ap0->n_items, (int)gridDim.x, ap0->n_queues}.first_item(blockIdx.x);
    empty_queues = 0;
  }
  for (;;) {
    // arguments and lane constants are read / derived anew for every item, so that nothing derived from them is
    // carried in registers across the item loop
    auto ap = (const __attribute__((address_space(4))) BwdArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
    const ItemQueues queues = {ap->ticket_slot, ap->n_items, (int)gridDim.x, ap->n_queues};
    __syncthreads();   // the previous item is done with LDS, and next_item[turn] has been written
    int w = __builtin_amdgcn_readfirstlane(next_item[turn]);
    turn ^= 1;
    if (w >= queues.n_items) {
      if (threadIdx.x == 0) queues.leave();
      break;
    }
    DkdvItemArgs a;
    a.q = ap->q; a.d_o = ap->d_o; a.lse = ap->lse; a.delta = ap->delta;
    a.bs = ap->bs; a.hq = ap->hq; a.hkv = ap->hkv; a.g = ap->g;
    a.Lq = ap->Lq; a.Lk = ap->Lk;
    a.n_tiles = ap->n_tiles; a.causal = ap->causal; a.heads_per_wg = ap->heads_per_wg;
    a.scale = ap->scale; a.scale_log2 = ap->scale_log2;
    a.qpos = PosDesc32{ap->qpos.start0, ap->qpos.len0, ap->qpos.start1, ap->qpos.len1};
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keep what derives from it in scalar registers
    const int l32 = lane & 31, hl = lane >> 5;
    const int n_groups = a.bs * a.hkv;
    const int group = w % n_groups; w /= n_groups;
    const int n_hsplit = a.g / a.heads_per_wg;   // workgroups that share a key tile's outputs (1: nobody else)
    const int hsplit = w % n_hsplit; w /= n_hsplit;
    const int hg0 = hsplit * a.heads_per_wg;
    const int q_splits = ap->q_splits;
    const int qs = w % q_splits; w /= q_splits;   // this item's slice of the visible query tiles
    const int ktile = w % a.n_tiles;         // ascending local index: keys seen by the most queries first
    const int blk = w / a.n_tiles;           // K/V block of the ring loop
    const PosDesc32 kpos = {ap->kpos[blk].start0, ap->kpos[blk].len0, ap->kpos[blk].start1, ap->kpos[blk].len1};
    const int b = group / a.hkv, kvh = group % a.hkv;
    const int tile_key0 = ktile * BN, tile_key1 = min(a.Lk, tile_key0 + BN);
    const int wave_key0 = tile_key0 + wave * 32;
    const int key = wave_key0 + l32;
    const int kk = min(key, a.Lk - 1);
    const int kp = a.causal ? pos_of(kpos, kk) : 0;
    const bool key_ok = key < a.Lk;

    // B operands of S = Q K^T and dP = dO V^T: lane = key l32, dims 16 ks + 8 hl ..  The K fragments stay in
    // registers; the V fragments are read from LDS every step (both in registers next to the two accumulators
    // do not fit 256 VGPRs: the spills' reloads share the counter of the prefetch loads and stall on them).
    bf16x8 kf[KSTEPS];
    {
      const size_t off = (((size_t)b * a.Lk + kk) * a.hkv + kvh) * HS + 8 * hl;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) kf[ks] = *(const bf16x8*)((const __bf16*)ap->k[blk] + off + 16 * ks);
      const char* vg = (const char*)((const __bf16*)ap->v[blk] + ((size_t)b * a.Lk * a.hkv + kvh) * HS);
      const uint32_t v_row_bytes = (uint32_t)a.hkv * HS * 2;
#pragma unroll
      for (int c = 0; c < BN * CPR / NT; ++c) {
        const int r = (tid + c * NT) / CPR, col = (tid + c * NT) % CPR;
        const int krow = min(tile_key0 + r, a.Lk - 1);
        *(u32x4*)(v_s + r * USTR + col * 16) = *(const u32x4*)(vg + (size_t)krow * v_row_bytes + col * 16);
      }
    }
    const char* v_row = v_s + (wave * 32 + l32) * USTR + hl * 16;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) settle(kf[ks]);
    f32x16 dk[DB], dv[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      zero16(dk[db]);
      zero16(dv[db]);
    }

    const TileRanges tr = visible_query_tiles<QT>(a.causal, a.qpos, kpos, a.Lq, tile_key0, tile_key1);
    const int na = tr.a1 - tr.a0, nt = na + (tr.b1 - tr.b0);
    // Query tiles are walked from the LAST one down: every workgroup of a head then starts on the same tile and
    // the ones running side by side on an XCD read the same Q / dO rows at about the same time (one L2 fill
    // serves them all); walking up from each workgroup's own diagonal would spread them over the sequence.
    auto tile_of = [&](int it) { const int j = nt - 1 - it; return j < na ? tr.a0 + j : tr.b0 + (j - na); };
    const bool wave_live = wave_key0 < a.Lk;
    const int wave_kmax = (a.causal && wave_live) ? pos_max(kpos, wave_key0, min(a.Lk, wave_key0 + 32)) : 0;
    // Query tiles this wave need not mask: full tiles that lie wholly in one ascending run of the query positions
    // and whose first row none of the wave's keys follows (and only if the wave's 32 keys all exist).  As places
    // j in the visible ranges (tile_of(it) is place nt - 1 - it) they are [free_a0, free_a1) and [free_b0, free_b1),
    // worked out here once per work item; the decision per tile is then a few comparisons.
    int free_a0 = 0, free_a1 = 0, free_b0 = 0, free_b1 = 0;
    if (wave_live && wave_key0 + 32 <= a.Lk) {
      const int full = a.Lq / QT;
      int ta0 = 0, ta1 = full, tb0 = 0, tb1 = 0;   // as tile numbers
      if (a.causal) {
        int64_t g0 = (int64_t)wave_kmax - a.qpos.start0; g0 = g0 < 0 ? 0 : (g0 > a.qpos.len0 ? a.qpos.len0 : g0);
        int64_t g1 = (int64_t)wave_kmax - a.qpos.start1; g1 = g1 < 0 ? 0 : (g1 > a.qpos.len1 ? a.qpos.len1 : g1);
        ta0 = (int)((g0 + QT - 1) / QT);
        ta1 = min(full, a.qpos.len0 / QT);
        tb0 = (int)(((int64_t)a.qpos.len0 + g1 + QT - 1) / QT);
        tb1 = min(full, (int)(((int64_t)a.qpos.len0 + a.qpos.len1) / QT));
      }
      free_a0 = max(ta0, tr.a0) - tr.a0;
      free_a1 = min(ta1, tr.a1) - tr.a0;
      free_b0 = na + max(max(tb0, ta1), tr.b0) - tr.b0;
      free_b1 = na + min(tb1, tr.b1) - tr.b0;
    }

    const int st_row = tid / CPR, st_col = tid % CPR;
    const bool stager = st_row < QT;
    u32x4 qreg, oreg;
    float streg = 0.f;
    // tile base addresses are wave-uniform; the per-thread byte offset is the same for every tile, clamped by a
    // min on the offset for rows past the last query (offsets grow with the row)
    const uint32_t row_bytes = (uint32_t)a.hq * HS * 2;
    const uint32_t st_off = (uint32_t)st_row * row_bytes + st_col * 16;
    const char* qg = nullptr;      // per query head, set at the top of the head loop
    const char* og = nullptr;
    const float* stat_g = nullptr;
    const float inv_scale = 1.0f / a.scale;
    auto fetch = [&](int it) {
      const int q0 = tile_of(it) * QT;
      if (stager) {
        const uint32_t lim = (uint32_t)min(a.Lq - 1 - q0, QT - 1) * row_bytes + st_col * 16;
        const uint32_t off = min(st_off, lim);
        qreg = *(const u32x4*)(qg + (size_t)q0 * row_bytes + off);
        oreg = *(const u32x4*)(og + (size_t)q0 * row_bytes + off);
      }
      if (tid < 2 * QT) streg = stat_g[min(q0 + (tid % QT), a.Lq - 1)];   // raw: converted when stashed, not here
    };
    auto stash = [&](int buf) {
      char* base = lds + buf * STAGE;
      if (stager) {
        *(u32x4*)(base + st_row * USTR + st_col * 16) = qreg;
        *(u32x4*)(base + QT * USTR + st_row * USTR + st_col * 16) = oreg;
      }
      if (tid < 2 * QT) {
        // The row statistics ride through the matrix core: with one more k-step whose A row is x split into three
        // bf16 pieces (exact to fp32 accuracy) and whose B column is 1, 1, 1, the first product comes out as
        // q.k - LSE/scale (threads 0..QT-1, into the Q rows) and dO.v - D (the next QT threads, into the dO rows)
        // without any per-row read by the 16 rows a lane holds.  A row that saw nothing gets -1e30: P = 0.
        float x = tid < QT ? ((streg == -INFINITY) ? -1e30f : fmaxf(fminf(-streg * inv_scale, 1e30f), -1e30f)) : -streg;
        const __bf16 hi = (__bf16)x;
        x -= (float)hi;
        const __bf16 mid = (__bf16)x;
        x -= (float)mid;
        const __bf16 lo = (__bf16)x;
        const bf16x8 piece = {hi, mid, lo, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
        *(bf16x8*)(base + (tid < QT ? 0 : QT * USTR) + (tid % QT) * USTR + XOFF) = piece;
      }
    };
    const int tr_off = tr_lane_offset<USTR>(lane);
    const int row_off = l32 * USTR + hl * 16;
    // The query heads of the KV group that this workgroup walks (all g of them when the grid is large enough
    // without splitting them: then nobody else adds to these keys' dK/dV and the epilogue is a plain store).
    for (int hh = 0; hh < a.heads_per_wg; ++hh) {
    const int h = kvh * a.g + hg0 + hh;
    qg = (const char*)((const __bf16*)a.q + ((size_t)b * a.Lq * a.hq + h) * HS);
    og = (const char*)((const __bf16*)a.d_o + ((size_t)b * a.Lq * a.hq + h) * HS);
    stat_g = (tid < QT ? a.lse : a.delta) + ((size_t)b * a.hq + h) * a.Lq;
    const int it0 = (int)((int64_t)nt * qs / q_splits), it1 = (int)((int64_t)nt * (qs + 1) / q_splits);
    // where the dS blocks of this head and K/V block begin
    char* ds_head = nullptr;
    const int ds_lane_off = l32 * 32 + hl * 16;
    if constexpr (WRITE_DS)
      ds_head = (char*)ap->ds + ((((size_t)b * a.hq + h) * ap->n_blocks + blk) * ap->ds_qt8 * ap->ds_kt * 8) * 2048;
    if (it1 > it0) {
      fetch(it0);
      stash(it0 & 1);   // the previous head's last step ended on a barrier
    }
    __syncthreads();
    for (int it = it0; it < it1; ++it) {
      const bool more = it + 1 < it1;
      const char* base = lds + (it & 1) * STAGE;
      const char* q_s = base;
      const char* o_s = base + QT * USTR;
      const int q0 = tile_of(it) * QT;

      // S = Q K^T and dP = dO V^T: rows = queries, cols = keys
      // Operand reads run ahead of the products that use them (read just in time, every product waited out a full LDS
      // latency): the Q fragment of k-step ks + 1 is read before the S product of ks (two registers sets), the dO and V
      // fragments of ks + 1 right after the dP product of ks has taken its operands (one set).  Three full sets do
      // not fit: the prefetched Q rows were spilled, with a wait for the global load on the spot.
      f32x16 s, dp;
      zero16(s);
      zero16(dp);
      bf16x8 qa[2], oa, vb;
      qa[0] = *(const bf16x8*)(q_s + row_off);
      oa = *(const bf16x8*)(o_s + row_off);
      vb = *(const bf16x8*)(v_row);
      // the extra k-step's B operand (k indices 0..2 one, the rest zero), made anew in every step from a lane index
      // the compiler cannot see through: kept across the loop it is four more registers
      bf16x8 ones_now;
      {
        int hz = hl;
        asm volatile("" : "+v"(hz));
        const u32x4 w = {hz == 0 ? 0x3F803F80u : 0u, hz == 0 ? 0x00003F80u : 0u, 0u, 0u};
        ones_now = __builtin_bit_cast(bf16x8, w);
      }
#pragma unroll
      for (int ks = 0; ks <= KSTEPS; ++ks) {
        const int cur = ks & 1, nxt = cur ^ 1;
        // k-step KSTEPS is the extra one (row statistics: s -= LSE / scale, dp -= D): its A rows lie in the padding
        if (ks < KSTEPS) qa[nxt] = *(const bf16x8*)(q_s + row_off + (ks + 1 < KSTEPS ? (ks + 1) * 32 : XOFF));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[cur], ks < KSTEPS ? kf[ks < KSTEPS ? ks : 0] : ones_now, s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(oa, ks < KSTEPS ? vb : ones_now, dp, 0, 0, 0);
        if (ks < KSTEPS) {
          oa = *(const bf16x8*)(o_s + row_off + (ks + 1 < KSTEPS ? (ks + 1) * 32 : XOFF));
          if (ks + 1 < KSTEPS) vb = *(const bf16x8*)(v_row + (ks + 1) * 32);
        }
      }
      // pin that order (left alone, the scheduler pulls every read back to just before its product to save registers)
      __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
      for (int ks = 0; ks + 1 < KSTEPS; ++ks) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);

      // The next tile's rows are fetched HERE, not at the top of the step: the first 18 products are where the
      // registers run out (the operand reads cannot be issued ahead), and the two prefetch registers are not live there.
      __builtin_amdgcn_sched_barrier(0);
      if (more) fetch(it + 1);
      __builtin_amdgcn_sched_barrier(0);

      // this lane: key column l32; register i <-> query row 8 (i/4) + 4 hl + (i%4) of the tile.
      // P and dS overwrite s and dp in place; the mask (rare: tiles on the causal boundary or ragged) sits
      // behind a wave-uniform branch.
      const int jq = nt - 1 - it;   // the tile's place in the visible ranges
      const bool need_mask = !((jq >= free_a0 && jq < free_a1) || (jq >= free_b0 && jq < free_b1));
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = __builtin_amdgcn_exp2f(s[i] * a.scale_log2);
      if (need_mask) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int qr = q0 + 8 * (i >> 2) + 4 * hl + (i & 3);
          const bool vis = qr < a.Lq && key_ok && (!a.causal || kp <= pos_of(a.qpos, qr));
          s[i] = vis ? s[i] : 0.f;
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) dp[i] *= s[i];

      __amdgpu_buffer_rsrc_t ds_blk;   // this wave's block of dS for this query tile
      if constexpr (WRITE_DS) {
        const int qt = q0 / QT;
        const size_t idx = ((size_t)(qt >> 3) * ap->ds_kt + (ktile * 8 + wave)) * 8 + (qt & 7);
        ds_blk = __builtin_amdgcn_make_buffer_rsrc(ds_head + idx * 2048, 0, 2048, kRawBufferFlags);
      }
      // dV^T += dO^T P and dK^T += Q^T dS   (rows = head dims, cols = keys, k = queries)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        u32x4 pw, dw;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
          pw[pr] = pack_bf16(s[8 * st + 2 * pr], s[8 * st + 2 * pr + 1]);
          dw[pr] = pack_bf16(dp[8 * st + 2 * pr], dp[8 * st + 2 * pr + 1]);
        }
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw), dsf = __builtin_bit_cast(bf16x8, dw);
        if constexpr (WRITE_DS) {
          // dw holds query rows 16 st + 4 hl .. + 3 and 8 more on .. + 3 of key column l32.  The two lanes of a key
          // trade halves (v_permlane32_swap(a, b): lower lanes get {a, a of lane + 32}, upper lanes {b of lane - 32,
          // b}), so that the lower one holds rows 16 st .. + 7 and the upper one rows 16 st + 8 .. + 15: 16 bytes each
          const u32x2 e = __builtin_amdgcn_permlane32_swap(dw[0], dw[2], false, false);
          const u32x2 o = __builtin_amdgcn_permlane32_swap(dw[1], dw[3], false, false);
          // The block's address is in the descriptor and the scalar offset stays an immediate zero: a buffer
          // store of more than 8 bytes reads its data registers after it has issued, and the compiler keeps the
          // next instructions from overwriting them only in this form.  (With the block's offset in a scalar
          // register, the data registers were reused at once and some blocks came out holding the next step's
          // values, now and then: measured, the results differed from run to run.)
          __builtin_amdgcn_raw_buffer_store_b128(u32x4{e[0], o[0], e[1], o[1]}, ds_blk, ds_lane_off + 1024 * st, 0, kDsStoreAux);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 ot = tr_read<USTR>(o_s + tr_off + (16 * st) * USTR + db * 64);
          const bf16x8 qt = tr_read<USTR>(q_s + tr_off + (16 * st) * USTR + db * 64);
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ot, pf, dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, dsf, dk[db], 0, 0, 0);
        }
      }
      // Here too the transpose reads of the next pair of products may be asked to go before the current pair (the
      // registers of S and dP are free by now).  Measured side by side: the instance that writes dS gains 1.4 % of the
      // whole backward, the plain one loses 0.4-0.9 % (its schedule comes out differently): only the former asks.
      if constexpr (WRITE_DS) {
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int i = 0; i < 2 * DB - 1; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
      if (more) stash((it + 1) & 1);
      __syncthreads();
    }
    }   // query heads

    unsigned own_ticket = kNoDraw;
    if (threadIdx.x == 0) own_ticket = queues.begin(empty_queues);
    if (key_ok) {
      const size_t part_stride = ap->dkdv_part_stride;   // > 0: every (head split, query slice) has its own copy
      const size_t off = (size_t)(hsplit * q_splits + qs) * part_stride + (((size_t)b * a.Lk + key) * a.hkv + kvh) * HS + 4 * hl;
      float* dkp = ap->dk[blk] + off;
      float* dvp = ap->dv[blk] + off;
      if (n_hsplit > 1 && part_stride == 0) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
              atomicAdd(dkp + db * 32 + j * 8 + tt, dk[db][4 * j + tt] * a.scale);
              atomicAdd(dvp + db * 32 + j * 8 + tt, dv[db][4 * j + tt]);
            }
      } else {
        const bool add = ap->acc_dkdv[blk] != 0;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            f32x4 k4 = {dk[db][4 * j] * a.scale, dk[db][4 * j + 1] * a.scale, dk[db][4 * j + 2] * a.scale,
                        dk[db][4 * j + 3] * a.scale};
            f32x4 v4 = {dv[db][4 * j], dv[db][4 * j + 1], dv[db][4 * j + 2], dv[db][4 * j + 3]};
            f32x4* kd = (f32x4*)(dkp + db * 32 + j * 8);
            f32x4* vd = (f32x4*)(dvp + db * 32 + j * 8);
            if (add) {
              k4 += *kd;
              v4 += *vd;
            }
            *kd = k4;
            *vd = v4;
          }
      }
    }

    if (threadIdx.x == 0) {
      unsigned empty = empty_queues;
      next_item[turn] = queues.finish(own_ticket, empty);
      empty_queues = empty;
    }
  }   // next work item
}

__global__ __launch_bounds__(256) void bwd_zero_kernel(f32x4* dst, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n4) dst[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// Where the converted tensor goes when that is not the dense [bs, rows, heads, hs] it comes from but the sequence-layout
// shards of the rank's Ulysses group ([U][bs][rows_per_shard][seq_heads][hs], dst = the group's first shard, the
// rank's heads from head0 on): Algorithm 1's reverse all-to-all rides on the conversion's stores.  rows_per_shard = 0: dense.
struct ConvertSeq { int rows_per_shard = 0, seq_heads = 0, head0 = 0, heads = 0, hs4 = 0, bs = 0; int64_t rows = 0; };

// fp32 accumulator -> bf16 / fp32 output, 4 elements per lane; blockIdx.y picks one of two tensors of the same size
// (dK and dV go through one launch)
template <typename OutT>
__global__ __launch_bounds__(256) void bwd_convert_kernel(const float* src0, OutT* dst0, const float* src1, OutT* dst1,
                                                          size_t n4, int n_copies, size_t copy_stride4, int add_to_dst,
                                                          ConvertSeq cs) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const float* src = blockIdx.y ? src1 : src0;
  OutT* dst = blockIdx.y ? dst1 : dst0;
  f32x4 v = __builtin_nontemporal_load((const f32x4*)src + i);
  for (int c = 1; c < n_copies; ++c) v += __builtin_nontemporal_load((const f32x4*)src + c * copy_stride4 + i);
  size_t o = i;   // in groups of four elements
  if (cs.rows_per_shard) {
    const size_t e4 = i % cs.hs4, rh = i / cs.hs4;
    const size_t h = rh % cs.heads, br = rh / cs.heads;
    const size_t row = br % cs.rows, b = br / cs.rows;
    const size_t shard = row / cs.rows_per_shard, sr = row - shard * cs.rows_per_shard;
    o = (((shard * cs.bs + b) * cs.rows_per_shard + sr) * cs.seq_heads + cs.head0 + h) * cs.hs4 + e4;
  }
  if constexpr (sizeof(OutT) == 4) {
    if (add_to_dst) v += *((const f32x4*)dst + o);
    __builtin_nontemporal_store(v, (f32x4*)dst + o);
  } else {
    u32x2 pk = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
    __builtin_nontemporal_store(pk, (u32x2*)dst + o);
  }
}

template <int HS, bool WRITE_DS>
int launch_dkdv(const BwdArgs& a, int64_t grid, hipStream_t stream) {
  constexpr int USTR = HS * 2 + 48;
  constexpr size_t lds = 256 * USTR + 2 * (2 * 32 * USTR);
  static LdsLimitRaised lds_limit;   // per kernel instance
  if (!raise_dynamic_lds_limit((const void*)bwd_dkdv_kernel<HS, WRITE_DS>, lds, lds_limit)) return USP_ERR_LAUNCH;
  hipLaunchKernelGGL((bwd_dkdv_kernel<HS, WRITE_DS>), dim3((unsigned)grid), dim3(512), lds, stream, a);
  return launch_status();
}

template <int HS>
int launch_dq_ds(const BwdArgs& a, int64_t grid, hipStream_t stream) {
  constexpr int KT = 128;
  constexpr int USTR = HS * 2 + 48;
  constexpr size_t lds = 2 * KT * USTR + 8 * (KT / 32) * kDsBlockLds;
  static LdsLimitRaised lds_limit;   // per kernel instance
  if (!raise_dynamic_lds_limit((const void*)bwd_dq_ds_kernel<HS, KT>, lds, lds_limit)) return USP_ERR_LAUNCH;
  hipLaunchKernelGGL((bwd_dq_ds_kernel<HS, KT>), dim3((unsigned)grid), dim3(512), lds, stream, a);
  return launch_status();
}

}  // namespace

int launch_bwd_delta(const void* o, const void* d_o, float* delta, int bs, int64_t L, int h, int hs,
                     hipStream_t stream, const SeqLayoutIO* seq) {
  const int seq_n = seq ? seq->rows_per_shard : 0, seq_heads = seq ? seq->heads : 0, seq_head0 = seq ? seq->head0 : 0;
  const int64_t rows = (int64_t)bs * L * h;
  const int tpr = hs / 8;
  const int64_t grid = (rows * tpr + 255) / 256;
  if (grid > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
  if (hs == 128)
    hipLaunchKernelGGL((bwd_delta_kernel<128>), dim3((unsigned)grid), dim3(256), 0, stream, (const __bf16*)o,
                       (const __bf16*)d_o, delta, bs, (int)L, h, seq_n, seq_heads, seq_head0);
  else
    hipLaunchKernelGGL((bwd_delta_kernel<64>), dim3((unsigned)grid), dim3(256), 0, stream, (const __bf16*)o,
                       (const __bf16*)d_o, delta, bs, (int)L, h, seq_n, seq_heads, seq_head0);
  return launch_status();
}

// How a launch pair divides its work.  dK/dV: one workgroup per (key tile, KV head, batch, block) that walks all g
// query heads of the group writes its outputs once; when that grid would leave CUs idle, the heads are split over
// workgroups, in the coarsest split that still gives every CU about four workgroups (a wide group, as in multi-query
// attention, would otherwise pay g-fold for meeting again), else one head per workgroup.  With room for copies of
// the outputs (`cut_items`) the items are divided further where that pays (measured on one rank of L = 8192 ... 65536):
// fewer than two dQ items per CU, each as long as its query tile has visible keys, are cut into slices of their key
// tiles until there are two per CU (at most 4 slices, of at least 32 tiles of 32 keys); fewer than two dK/dV items
// per CU likewise into slices of their query tiles (at least 16 tiles of 32 rows), and up to eight per CU into two
// slices when an item walks several heads (long items, few copies); one head per item and two or more items per CU
// are left alone (config 2: 8 copies of dK/dV instead of 4 cost 1 %).
BwdCut plan_bwd_cut(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int n_blocks, bool cut_items, bool equal_items) {
  BwdCut c;
  const int g = hq / hkv;
  const int64_t unsplit = ((Lk + 255) / 256) * hkv * bs * n_blocks;
  c.heads_per_wg = g;
  if (unsplit < 2 * kPlanCUs) {
    c.heads_per_wg = 1;
    for (int h = g - 1; h > 1; --h)
      if (g % h == 0 && unsplit * (g / h) >= 4 * kPlanCUs) { c.heads_per_wg = h; break; }
  }
  c.k_splits = c.q_splits = 1;
  if (cut_items) {
    const int64_t dq_items = ((Lq + 255) / 256) * hq * bs;
    const int64_t key_tiles = (int64_t)n_blocks * ((Lk + 31) / 32), query_tiles = (Lq + 31) / 32;
    if (dq_items < 2 * kPlanCUs)
      c.k_splits = (int)std::max<int64_t>(1, std::min<int64_t>({4, (2 * kPlanCUs + dq_items - 1) / dq_items, key_tiles / 32}));
    const int64_t dkdv_items = unsplit * (g / c.heads_per_wg);
    if (dkdv_items < 2 * kPlanCUs)
      c.q_splits = (int)std::max<int64_t>(1, std::min<int64_t>({4, (2 * kPlanCUs + dkdv_items - 1) / dkdv_items, query_tiles / 16}));
    else if (dkdv_items < 8 * kPlanCUs && c.heads_per_wg > 1)
      c.q_splits = (int)std::max<int64_t>(1, std::min<int64_t>(2, query_tiles / 16));
    if (equal_items) {
      // Without a mask every item of a kernel weighs the same and the time is rounds of kPlanCUs items: s slices make
      // ceil(items x s / CUs) rounds of 1/s each (320 items: 2, 1.5, 1.33, 1.25 for 1 ... 4 slices).  The fewest slices
      // within 3 % of the best, each further slice charged 2 % for its copy of the output (measured, one rank of four
      // heads: L = 12288 1.22 -> 1.06 ms with 4 + 4 slices instead of 2 + 2, L = 20480 2.95 -> 2.73, L = 28672 5.39 -> 5.20).
      auto slices = [](int64_t items, int64_t max_slices) {
        int best = 1;
        double best_t = 1e30;
        for (int s = 1; s <= max_slices; ++s) {
          const double t = (double)((items * s + kPlanCUs - 1) / kPlanCUs) / s * (1.0 + 0.02 * (s - 1));
          if (t < 0.97 * best_t) { best = s; best_t = t; }
        }
        return best;
      };
      c.k_splits = slices(dq_items, std::max<int64_t>(1, std::min<int64_t>(4, key_tiles / 32)));
      c.q_splits = slices(dkdv_items, std::max<int64_t>(1, std::min<int64_t>(4, query_tiles / 16)));
    }
  }
  return c;
}

int launch_ring_attn_bwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                         const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks, int bs,
                         int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                         const usp_posdesc& qpos, int accumulate_dq, const int* accumulate_dkdv,
                         hipStream_t stream, const BwdCopies* copies) {
  if (n_blocks < 1 || n_blocks > kMaxBlocks) return USP_ERR_UNSUPPORTED;
  // without room for copies: items are not cut, and heads that are split over workgroups meet through atomic adds
  const BwdCut cut = copies ? copies->cut : plan_bwd_cut(bs, Lq, Lk, hq, hkv, n_blocks, false, false);
  BwdArgs a;
  a.k_splits = cut.k_splits;
  a.q_splits = cut.q_splits;
  a.dq_part_stride = copies ? copies->dq_stride : 0;
  a.dkdv_part_stride = copies ? copies->dkdv_stride : 0;
  a.q = q; a.d_o = d_o; a.lse = lse; a.delta = delta;
  a.dq = dq;
  for (int j = 0; j < kMaxBlocks; ++j) {
    const int jj = j < n_blocks ? j : 0;
    a.k[j] = k_blocks[jj];
    a.v[j] = v_blocks[jj];
    a.dk[j] = dk_blocks[jj];
    a.dv[j] = dv_blocks[jj];
    const usp_posdesc& kp = kpos_blocks[jj];
    a.kpos[j] = PosDesc32{(int)kp.start0, (int)kp.len0, (int)kp.start1, (int)kp.len1};
  }
  a.n_blocks = n_blocks;
  a.bs = bs; a.hq = hq; a.hkv = hkv; a.g = hq / hkv;
  a.Lq = (int)Lq; a.Lk = (int)Lk;
  a.causal = causal;
  a.accumulate = accumulate_dq;
  a.scale = scale;
  a.scale_log2 = scale * kLog2e;
  a.qpos = PosDesc32{(int)qpos.start0, (int)qpos.len0, (int)qpos.start1, (int)qpos.len1};
  a.ds = copies ? copies->ds : nullptr;
  a.ds_kt = (int)((Lk + 255) / 256) * 8;
  a.ds_qt8 = (int)((Lq + 255) / 256);
  auto launch_dq = [&]() -> int {
    a.n_tiles = (a.Lq + 255) / 256;
    const int64_t grid = (int64_t)a.n_tiles * hq * bs * a.k_splits;
    if (grid > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
    // one workgroup per CU (256 VGPRs x 8 waves fill it), fewer when there are fewer items
    a.ticket_slot = ticket_slot_for(stream);
    a.n_items = (int)grid;
    a.n_queues = std::gcd(dev::kMaxItemQueues, bs * hkv);
    const unsigned n_wgs = (unsigned)std::min<int64_t>(grid, compute_units());
    int st;
    if (a.ds) {
      st = hs == 128 ? launch_dq_ds<128>(a, n_wgs, stream) : launch_dq_ds<64>(a, n_wgs, stream);
    } else {
      if (hs == 128)
        hipLaunchKernelGGL((bwd_dq_kernel<128>), dim3(n_wgs), dim3(512), 0, stream, a);
      else
        hipLaunchKernelGGL((bwd_dq_kernel<64>), dim3(n_wgs), dim3(512), 0, stream, a);
      st = launch_status();
    }
    return st;
  };
  auto launch_dkdv_pair = [&]() -> int {
    a.n_tiles = (a.Lk + 255) / 256;
    const int64_t unsplit = (int64_t)a.n_tiles * hkv * bs * n_blocks;
    a.heads_per_wg = cut.heads_per_wg;
    for (int j = 0; j < kMaxBlocks; ++j) a.acc_dkdv[j] = accumulate_dkdv[j < n_blocks ? j : 0];
    if (a.heads_per_wg != a.g && !copies) {   // atomic adds need accumulators that start from zero
      const size_t n4 = (size_t)bs * Lk * hkv * hs / 4;
      const size_t zg = (n4 + 255) / 256;
      if (zg > 0x7fffffffull) return USP_ERR_UNSUPPORTED;
      for (int j = 0; j < n_blocks; ++j) {
        if (accumulate_dkdv[j]) continue;
        hipLaunchKernelGGL(bwd_zero_kernel, dim3((unsigned)zg), dim3(256), 0, stream, (f32x4*)dk_blocks[j], n4);
        hipLaunchKernelGGL(bwd_zero_kernel, dim3((unsigned)zg), dim3(256), 0, stream, (f32x4*)dv_blocks[j], n4);
      }
    }
    const int64_t grid = unsplit * (a.g / a.heads_per_wg) * a.q_splits;
    if (grid > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
    // one workgroup per CU (256 VGPRs x 8 waves fill it), fewer when there are fewer items
    a.ticket_slot = ticket_slot_for(stream);
    a.n_items = (int)grid;
    // workgroups that walk the same query head share its Q / dO rows through the XCD's L2: one queue per
    // (KV group, head split) value, the two fastest indices of the item number
    a.n_queues = std::gcd(dev::kMaxItemQueues, bs * hkv * (a.g / a.heads_per_wg));
    const int64_t n_wgs = std::min<int64_t>(grid, compute_units());
    return a.ds ? (hs == 128 ? launch_dkdv<128, true>(a, n_wgs, stream) : launch_dkdv<64, true>(a, n_wgs, stream))
                : (hs == 128 ? launch_dkdv<128, false>(a, n_wgs, stream) : launch_dkdv<64, false>(a, n_wgs, stream));
  };
  // with dS kept, the dK/dV kernel (which writes it) runs first; otherwise the two are independent
  int st = a.ds ? launch_dkdv_pair() : launch_dq();
  if (st != USP_OK) return st;
  st = a.ds ? launch_dq() : launch_dkdv_pair();
  if (st != USP_OK) return st;
  return launch_status();
}

int launch_block_attn_bwd(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                          const float* delta, float* dq, float* dk, float* dv, int bs, int64_t Lq, int64_t Lk, int hq,
                          int hkv, int hs, float scale, int causal, const usp_posdesc& qpos, const usp_posdesc& kpos,
                          int accumulate_dq, int accumulate_dkdv, hipStream_t stream) {
  return launch_ring_attn_bwd(q, &k, &v, &kpos, 1, d_o, lse, delta, dq, &dk, &dv, bs, Lq, Lk, hq, hkv, hs, scale,
                              causal, qpos, accumulate_dq, &accumulate_dkdv, stream);
}

int launch_bwd_convert(const float* src, void* dst, size_t n, int out_dtype, hipStream_t stream, int n_copies,
                       size_t copy_stride, int add_to_dst) {
  return launch_bwd_convert2(src, dst, nullptr, nullptr, n, out_dtype, stream, n_copies, copy_stride, add_to_dst);
}

int launch_bwd_convert2(const float* src0, void* dst0, const float* src1, void* dst1, size_t n, int out_dtype,
                        hipStream_t stream, int n_copies, size_t copy_stride, int add_to_dst) {
  return launch_bwd_convert_seq(src0, dst0, src1, dst1, n, out_dtype, stream, n_copies, copy_stride, add_to_dst, nullptr,
                                0, 0, 0, 0);
}

int launch_bwd_convert_seq(const float* src0, void* dst0, const float* src1, void* dst1, size_t n, int out_dtype,
                           hipStream_t stream, int n_copies, size_t copy_stride, int add_to_dst, const SeqLayoutIO* seq,
                           int bs, int64_t rows, int heads, int hs) {
  ConvertSeq cs;
  if (seq) {
    if ((size_t)bs * rows * heads * hs != n || hs % 4) return USP_ERR_UNSUPPORTED;
    cs.rows_per_shard = seq->rows_per_shard; cs.seq_heads = seq->heads; cs.head0 = seq->head0;
    cs.heads = heads; cs.hs4 = hs / 4; cs.bs = bs; cs.rows = rows;
  }
  if (add_to_dst && out_dtype != USP_FP32) return USP_ERR_UNSUPPORTED;
  const size_t n4 = n / 4;
  const size_t grid = (n4 + 255) / 256;
  if (grid > 0x7fffffffull || n_copies < 1 || (copy_stride & 3)) return USP_ERR_UNSUPPORTED;
  const dim3 g((unsigned)grid, src1 ? 2u : 1u);
  if (out_dtype == USP_FP32)
    hipLaunchKernelGGL((bwd_convert_kernel<float>), g, dim3(256), 0, stream, src0, (float*)dst0, src1, (float*)dst1, n4,
                       n_copies, copy_stride / 4, add_to_dst, cs);
  else
    hipLaunchKernelGGL((bwd_convert_kernel<__bf16>), g, dim3(256), 0, stream, src0, (__bf16*)dst0, src1, (__bf16*)dst1,
                       n4, n_copies, copy_stride / 4, 0, cs);
  return launch_status();
}

}  // namespace usp
