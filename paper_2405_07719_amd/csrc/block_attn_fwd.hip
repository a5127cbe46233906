// Blockwise attention (Sec. 2: SP-Ring's blockwise loop; Eq. 1 restricted to the K/V blocks given):
// S = scale * Q K^T -> position mask -> online softmax over key tiles -> P V, returning O (the partial O of
// one ring step, or the final O when the launch covers the whole ring loop) and the per-row log-sum-exp.
//
// gfx950 design (bf16 instance)
//   * MFMA v_mfma_f32_32x32x16_bf16, fp32 accumulation.  The score tile is computed TRANSPOSED,
//     S^T = K Q^T: a lane then owns one query column (lane % 32) and 16 keys per 32-key block in
//     its accumulator registers, so the softmax row max / row sum are in-register reductions plus
//     one exchange between lanes l and l^32.  The accumulator layout of S^T is also the B-operand
//     layout of the second product O^T = V^T P^T (same lane <-> query, 8 keys per 16-key step), so
//     P never leaves registers.
//   * A workgroup owns BM = NWAVES * NQB * 32 query rows of one (batch, head); Q fragments stay in
//     registers for the whole kernel.  K and V tiles of KT keys are staged in LDS, double
//     buffered, fetched to registers one tile ahead while the current tile is being multiplied.
//   * K is read from LDS as row-major 16 B fragments (A operand, rows = keys).  V stays row-major
//     in LDS too; the V^T A-operand (rows = head dims, k = keys) is produced by the LDS transpose
//     read ds_read_b64_tr_b16, which hands each lane 4 consecutive keys of its head dim.
//   * exp2 with log2(e) folded into the scale; masks only on tiles that straddle the causal
//     boundary or the ragged tail; key tiles that are invisible to the whole query tile are
//     never loaded; the O accumulator is rescaled only when some row maximum moved.
//   * One workgroup per CU, persistent: work items (query tile x head x batch) are drawn from
//     counters in device memory, heaviest query tiles first (descending local index under a
//     causal mask), KV group fastest; a workgroup prefers the items whose KV heads its XCD's L2
//     already serves (attn_device.h).  K/V tiles are fetched through buffer descriptors.
#include <numeric>
#include <type_traits>

#include "attn_device.h"
#include "usp_internal.h"

namespace usp {
namespace {

using namespace dev;

constexpr int kMaxBlocks = USP_MAX_RING_BLOCKS;

// One launch covers n_blocks K/V blocks of Lk keys each (the ring steps of one rank, Algorithm 1 step 5): the
// online-softmax state of a query row stays in registers from the first block to the last, so no partial results
// and no merge pass exist.  n_blocks = 1 is the plain single ring step.
struct AttnArgs {
  const void* q;
  const void* k[kMaxBlocks];
  const void* v[kMaxBlocks];
  void* o;
  float* lse;
  int bs, hq, hkv, g;
  int Lq, Lk;
  int n_qtiles;
  int n_blocks;
  int causal;
  float scale;        // natural-units scale (for the LSE)
  float scale_log2;   // scale * log2(e)
  PosDesc32 qpos;
  PosDesc32 kpos[kMaxBlocks];
  // Where Q rows are read and O rows written.  seq_n == 0: dense [bs,Lq,hq,hs] (the layout after the forward
  // all-to-all).  seq_n > 0: straight from / to the sequence-layout shards of the rank's Ulysses group,
  // [U][bs][seq_n][seq_heads][hs] with this rank's heads at seq_head0: the all-to-all of Q (Algorithm 1 step 2)
  // and of O (step 6) folded into the one read of Q and the one write of O that the kernel does anyway.
  int seq_n, seq_heads, seq_head0;
  int ticket_slot;   // counter the workgroups draw their work items from (MFMA kernel)
  int n_items;       // work items of the launch: query tiles x heads x batch
  int n_queues;      // gcd(8, batch x KV heads): item w waits in queue w mod n_queues
  // Key split (launch_attn_fwd_partials): an item is (query tile, head, batch, ONE block), the blocks may differ in
  // their number of keys, and the item's O (fp32, dense) and LSE go to the block's own partial result.  Otherwise
  // (per_block = 0) an item walks all blocks, every block holds Lk keys and the result goes to o / lse.
  int per_block;
  // Mixed launch (launch_attn_fwd_mixed, kernel instance MIXED): the first n_split_items items are (query tile, head,
  // batch, ONE block) items as above, over the n_split_tiles query tiles that come first in item order (the heaviest
  // under a causal mask), each with its partial result; the items after them are whole items over the other query
  // tiles, which walk all blocks and write o / lse.  Every block holds lk_blk[j] keys.
  int n_split_items, n_split_tiles;
  int lk_blk[kMaxBlocks];
  void* o_part[kMaxBlocks];
  float* lse_part[kMaxBlocks];
  // Running state of a ring that delivers its blocks one per call (launch_block_attn_fwd_state): the online-softmax
  // state of every query row (running maximum m, sum l, unnormalised O^T accumulator) in the kernel's own register
  // layout, one record of state_record_floats() per 32-row block of a (batch, head): read at the start of an item
  // unless state_first, written at its end instead of O and LSE unless state_last.  Null: no state (all other paths).
  float* state;
  int state_first, state_last;
};

// floats of one 32-row state record: the O^T accumulator (hs / 32 x 16 registers x 64 lanes), then m and l per lane
constexpr size_t state_record_floats(int hs) { return (size_t)(hs / 32) * 16 * 64 + 2 * 64; }

// The scalar arguments as one work item of the MFMA kernel sees them (read anew for every item, see the kernel).
struct ItemArgs {
  const void* q;
  void* o;
  float* lse;
  int bs, hq, hkv, g;
  int Lq, Lk;
  int n_qtiles;
  int n_blocks;
  int causal;
  float scale, scale_log2;
  PosDesc32 qpos;
  int seq_n, seq_heads, seq_head0;
};

// element offset of (batch b, local row, local head h) in the Q / O tensor
template <typename Args>
__device__ inline size_t qo_offset(const Args& a, int b, int row, int h, int hs) {
  if (a.seq_n == 0) return (((size_t)b * a.Lq + row) * a.hq + h) * hs;
  const int shard = row / a.seq_n, s = row - shard * a.seq_n;
  return ((((size_t)shard * a.bs + b) * a.seq_n + s) * a.seq_heads + a.seq_head0 + h) * hs;
}

// -------------------------------------------------------------------------------------------
// bf16 MFMA kernel, software pipelined: while the softmax of key tile j runs on the vector ALU,
// the matrix core already computes the scores of tile j+1, then P(j) V(j).
// -------------------------------------------------------------------------------------------
// VT: the V blocks come in key-tile-transposed layout (usp.h: USP_SEQ_TO_HEAD_VT): per (batch, KV head) tiles of 64
// keys stored [hs][64 keys], the keys of each group of 16 in the order 0-3, 8-11, 4-7, 12-15.  The A operand of
// O^T = V^T P^T (rows = head dims, 8 keys per lane) is then ONE 16-byte row read per product instead of two LDS
// transpose reads: 32 LDS reads per step and wave (the minimum: one fragment per product) instead of 48, and the
// LDS pipe, which issues a read every ~7 cycles whatever its width, was the busiest unit of the kernel.
template <int HS, int NQB, int NWAVES, int KT, int WPE, typename OutT, bool STATE = false, bool VT = false, bool MIXED = false>
__global__ __attribute__((amdgpu_flat_work_group_size(NWAVES * 64, NWAVES * 64), amdgpu_waves_per_eu(WPE, WPE)))
void block_attn_fwd_mfma(const AttnArgs) {
  static_assert(!STATE || NQB == 1, "the state record is laid out for one 32-row block per wave");
  static_assert(!MIXED || (!STATE && sizeof(OutT) == 2), "the mixed launch writes bf16 results and fp32 partials");
  static_assert(!VT || KT == 64, "the transposed V layout is made of 64-key tiles");
  constexpr int NT = NWAVES * 64;
  constexpr int BM = NWAVES * NQB * 32;
  constexpr int KSTEPS = HS / 16;          // MFMA k-steps of Q K^T
  constexpr int DB = HS / 32;              // 32-wide head-dim blocks of O^T
  constexpr int KB = KT / 32;              // 32-key blocks of S^T
  constexpr int PS = KT / 16;              // MFMA k-steps of P V
  constexpr int KSTR = HS * 2 + 48;        // LDS row stride of K in bytes: an odd number of 16 B chunks, no bank conflicts on the row reads
  // V rows: an odd multiple of 64 B, no bank conflicts on the transpose reads; transposed tiles: rows of KT keys
  // (128 B) padded to an odd number of 16 B chunks like the K rows
  constexpr int VSTR = VT ? KT * 2 + 16 : HS * 2 + 64;
  constexpr int KBYTES = KT * KSTR, VBYTES = VT ? HS * VSTR : KT * VSTR;
  constexpr int VT_TILE_BYTES = HS * KT * 2;   // one transposed tile in global memory: [HS][KT] bf16, contiguous
  constexpr int CHUNKS = KT * HS / 8;      // 16 B chunks per tile (K and V alike)
  constexpr int CPT = CHUNKS / NT;         // chunks per thread
  constexpr float kRescaleThreshold = 8.0f;   // in log2 units: P stays below 2^8
  static_assert(CHUNKS % NT == 0, "tile must split evenly over the workgroup");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* const kbuf = smem;                  // [2][KBYTES]
  char* const vbuf = smem + 2 * KBYTES;     // [2][VBYTES]

  // ---- persistent workgroups: one per CU, each draws work items until none is left.  Item order: KV group
  //      fastest, then head within group, then query tile (heavy first).
  // The next item is drawn when the current one reaches its epilogue (not earlier: an item taken long before it is
  // started is no longer the next one in line when it starts, which is what balances the CUs): thread 0 asks at
  // the start of the epilogue and reads the answer after it, so the latency of the draw hides behind the stores
  // of O.  The item's number waits in LDS, two slots in turn: the next number may be written while slower waves
  // still read the current one.
  __shared__ int next_item[2];
  __shared__ unsigned empty_queues;   // thread 0's record of the item queues it has found empty
  int turn = 0;
  if (threadIdx.x == 0) {
    auto ap0 = (const __attribute__((address_space(4))) AttnArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    // the first item is given, not drawn
    next_item[0] = ItemQueues{ap0->ticket_slot, ap0->n_items, (int)gridDim.x, ap0->n_queues}.first_item(blockIdx.x);
    empty_queues = 0;
  }
  for (;;) {
    // The kernel arguments are read anew for every item, through a pointer to the argument segment that the
    // compiler cannot see through.  Read once, everything derived from them (reciprocals of the item decode, strides,
    // flags) would be hoisted out of the item loop and held in scalar registers across it; there are not enough,
    // and the overflow goes to lanes of a vector register that the tile loop cannot spare.
    auto ap = (const __attribute__((address_space(4))) AttnArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ap));
    const int n_items = ap->n_items;
    __syncthreads();   // the previous item is done with LDS, and next_item[turn] has been written
    int w = __builtin_amdgcn_readfirstlane(next_item[turn]);
    turn ^= 1;
    if (w >= n_items) {
      if (threadIdx.x == 0) ItemQueues{ap->ticket_slot, n_items, (int)gridDim.x, ap->n_queues}.leave();
      break;
    }
    ItemArgs a;
    a.q = ap->q; a.o = ap->o; a.lse = ap->lse;
    a.bs = ap->bs; a.hq = ap->hq; a.hkv = ap->hkv; a.g = ap->g;
    a.Lq = ap->Lq; a.Lk = ap->Lk;
    a.n_qtiles = ap->n_qtiles; a.n_blocks = ap->n_blocks; a.causal = ap->causal;
    a.scale = ap->scale; a.scale_log2 = ap->scale_log2;
    a.qpos = PosDesc32{ap->qpos.start0, ap->qpos.len0, ap->qpos.start1, ap->qpos.len1};
    a.seq_n = ap->seq_n; a.seq_heads = ap->seq_heads; a.seq_head0 = ap->seq_head0;
    const int n_groups = a.bs * a.hkv;
    // The lane constants are derived anew for every item from a thread index the compiler cannot see through:
    // hoisted out of the item loop they would stay in registers across it, and the tile loop has none to spare.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keep what derives from it in scalar registers
    const int l32 = lane & 31, hl = lane >> 5;
    bool per_block = ap->per_block != 0;
    if constexpr (MIXED) {
      per_block = w < ap->n_split_items;     // the split items come first
      if (!per_block) w -= ap->n_split_items;
    }
    const int group = w % n_groups; w /= n_groups;
    const int hg = w % a.g;
    int t = w / a.g;
    int blk0 = 0, blk1 = a.n_blocks;         // the blocks this item walks
    if (per_block) {
      blk0 = t % a.n_blocks;
      blk1 = blk0 + 1;
      t /= a.n_blocks;
    } else if constexpr (MIXED) {
      t += ap->n_split_tiles;
    }
    // (a mixed launch counts its tiles from the last one down whatever the mask: its cut tiles are the last rows)
    const int qtile = (a.causal || MIXED) ? a.n_qtiles - 1 - t : t;
    const int b = group / a.hkv, kvh = group % a.hkv;
    const int h = kvh * a.g + hg;

    const int tile_row0 = qtile * BM;
    const int tile_row1 = min(a.Lq, tile_row0 + BM);
    const int wave_row0 = tile_row0 + wave * (NQB * 32);

    if constexpr (STATE) {
      // A middle step of a step-by-step ring in which this query tile sees no key of the block (under the zigzag
      // split half of a rank's rows see nothing of most blocks): the rows' state stays as it is, so it is neither
      // read nor written back, and the item ends here.  (The first step writes the initial state, the last one the
      // output: those walk every item.)
      if (!ap->state_first && !ap->state_last) {
        bool any = false;
        for (int blk = 0; blk < a.n_blocks; ++blk) {
          const PosDesc32 kp = {ap->kpos[blk].start0, ap->kpos[blk].len0, ap->kpos[blk].start1, ap->kpos[blk].len1};
          const TileRanges t = visible_key_tiles<KT>(a.causal, a.qpos, kp, a.Lk, tile_row0, tile_row1);
          any = any || (t.a1 - t.a0) + (t.b1 - t.b0) > 0;
        }
        if (!any) {   // workgroup-uniform
          if (threadIdx.x == 0) {
            const ItemQueues queues = {ap->ticket_slot, n_items, (int)gridDim.x, ap->n_queues};
            const unsigned own_ticket = queues.begin(empty_queues);
            unsigned empty = empty_queues;
            next_item[turn] = queues.finish(own_ticket, empty);
            empty_queues = empty;
          }
          continue;
        }
      }
    }

    const __bf16* qg = (const __bf16*)a.q;
    const size_t kv_head_off = ((size_t)b * a.Lk * a.hkv + kvh) * HS * 2;   // bytes; + key * hkv * HS * 2
    // transposed V: the tiles of (batch, KV head) are contiguous; a.Lk (the batch stride in rows) gives their number
    const size_t vt_head_off = ((size_t)b * a.hkv + kvh) * (size_t)((a.Lk + KT - 1) / KT) * VT_TILE_BYTES;
    int Lk_b = a.Lk;   // keys of the current block (a.Lk stays the batch stride of every block's tensors)

    // ---- Q fragments (B operand of S^T = K Q^T): lane = query l32, dims 16*ks + 8*hl .. +7
    bf16x8 qf[NQB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int rr = min(wave_row0 + qb * 32 + l32, a.Lq - 1);
      const __bf16* src = qg + qo_offset(a, b, rr, h, HS) + 8 * hl;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) qf[qb][ks] = *(const bf16x8*)(src + 16 * ks);
    }

    // per-block state of the tile walk (workgroup-uniform), set at the top of the block loop
    const char* kg = nullptr;
    const char* vg = nullptr;
    PosDesc32 kpos = {0, 0, 0, 0};
    TileRanges tr = {0, 0, 0, 0};
    int na = 0, nt = 0;
    int free_a = 0, free_b0 = 0, free_b1 = 0;   // walk positions [0, free_a) and [free_b0, free_b1): tiles this wave need not mask
    auto tile_of = [&](int it) { return it < na ? tr.a0 + it : tr.b0 + (it - na); };

    f32x16 oacc[NQB][DB];
    float m_run[NQB], l_run[NQB];
    float zero = 0.f;
    asm volatile("" : "+v"(zero));   // not a constant to the compiler: it would share one zeroed register tuple between items
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      m_run[qb] = -INFINITY;
      l_run[qb] = zero;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[qb][db][i] = zero;
    }

    // ---- running state of a step-by-step ring: this wave's record (one per 32-row block of the head)
    // (an instance of its own, STATE: in the plain instance the code below is not there at all)
    float* st_rec = nullptr;
    if constexpr (STATE) {
      float* const st = ap->state;
      {
        st_rec = st + ((((size_t)b * a.hq + h) * a.n_qtiles + qtile) * NWAVES + wave) * state_record_floats(HS);
        if (!ap->state_first) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const f32x4 v4 = *(const f32x4*)(st_rec + ((db * 4 + j) * 64 + lane) * 4);
#pragma unroll
              for (int e = 0; e < 4; ++e) oacc[0][db][4 * j + e] = v4[e];
            }
          m_run[0] = st_rec[DB * 16 * 64 + lane];
          l_run[0] = st_rec[DB * 16 * 64 + 64 + lane];
        }
      }
    }

    // wave-level bounds for the mask decision
    const int wave_row1 = min(a.Lq, wave_row0 + NQB * 32);
    const bool wave_live = wave_row0 < a.Lq;
    const int wave_qmin = (a.causal && wave_live) ? pos_min(a.qpos, wave_row0, wave_row1) : 0;

    // ---- staging: each thread moves CPT 16 B chunks of a K tile and of a V tile
    const int st_row = tid / (HS / 8), st_col = tid % (HS / 8);
    constexpr int ROWS_PER_PASS = NT / (HS / 8);
    u32x4 kreg[CPT], vreg[CPT];
    // Tiles are read through a buffer descriptor built per tile in scalar registers: base = the tile's first row
    // (this KV head), extent = up to the end of its last valid row.  Each thread adds a 32-bit byte offset that is
    // the same for every tile; rows past the last key (ragged final tile only) lie beyond the extent and read as
    // zeros (the mask hides those keys).  No 64-bit address arithmetic on the vector ALU, no clamping.
    const uint32_t row_bytes = (uint32_t)a.hkv * HS * 2;
    uint32_t st_off[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) st_off[c] = (uint32_t)(st_row + c * ROWS_PER_PASS) * row_bytes + st_col * 16;
    // (`tile` is the tile's number in the block, not its place in the walk; the extent is one of two values that
    // are worked out once per block: a full tile's, or that of the block's ragged last tile)
    int full_tiles = 0, full_extent = 0, ragged_extent = 0;
    auto fetch = [&](const char* base, int tile, u32x4* reg) {
      const char* tb = base + (uint64_t)((uint32_t)tile * KT) * row_bytes;
      const __amdgpu_buffer_rsrc_t tile_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          (void*)tb, 0, tile < full_tiles ? full_extent : ragged_extent, kRawBufferFlags);
#pragma unroll
      for (int c = 0; c < CPT; ++c) reg[c] = __builtin_amdgcn_raw_buffer_load_b128(tile_rsrc, (int)st_off[c], 0, 0);
    };
    auto stash = [&](char* buf, int stride, const u32x4* reg) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) *(u32x4*)(buf + (st_row + c * ROWS_PER_PASS) * stride + st_col * 16) = reg[c];
    };
    // transposed V tiles: 16 KiB (8 KiB at head size 64) contiguous in global memory, chunk c of the tile goes to
    // row c / 8 (a head dim), 16 B column c % 8 of the LDS tile
    auto fetch_vt = [&](const char* base, int tile, u32x4* reg) {
      const char* tb = base + (uint64_t)(uint32_t)tile * VT_TILE_BYTES;
      const __amdgpu_buffer_rsrc_t tile_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)tb, 0, VT_TILE_BYTES, kRawBufferFlags);
#pragma unroll
      for (int c = 0; c < CPT; ++c) reg[c] = __builtin_amdgcn_raw_buffer_load_b128(tile_rsrc, (tid + c * NT) * 16, 0, 0);
    };
    auto stash_vt = [&](char* buf, const u32x4* reg) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int ch = tid + c * NT;
        *(u32x4*)(buf + (ch >> 3) * VSTR + (ch & 7) * 16) = reg[c];
      }
    };
    auto fetch_v = [&](const char* base, int tile, u32x4* reg) {
      if constexpr (VT) fetch_vt(base, tile, reg); else fetch(base, tile, reg);
    };
    auto stash_v = [&](char* buf, const u32x4* reg) {
      if constexpr (VT) stash_vt(buf, reg); else stash(buf, VSTR, reg);
    };

    // ---- S^T = K Q^T for the tile in K buffer kb_ (rows = keys, cols = queries)
    auto qk = [&](const char* kb_, f32x16 (&sacc)[NQB][KB]) {
      const char* krow = kb_ + l32 * KSTR + hl * 16;
      // k-step outermost: consecutive MFMAs go to different accumulators (no back-to-back dependence)
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) {
          const bf16x8 kf = *(const bf16x8*)(krow + kbk * 32 * KSTR + ks * 32);
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) {
            if (ks == 0) {
              f32x16 z;
#pragma unroll
              for (int i = 0; i < 16; ++i) z[i] = 0.f;
              sacc[qb][kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][ks], z, 0, 0, 0);
            } else {
              sacc[qb][kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][ks], sacc[qb][kbk], 0, 0, 0);
            }
          }
        }
      }
    };

    // One pipeline step on tile `it` whose scores are in s_cur.  Unless LAST, the scores of tile it+1
    // are produced into s_next while the softmax of s_cur runs.
    int v_tile = 0;   // number of the V tile the next step prefetches (workgroup-uniform)
    const int grp = lane >> 4, j16 = lane & 15;
    const int v_lane_off = (4 * hl + (j16 >> 2)) * VSTR + (16 * (grp & 1) + 4 * (j16 & 3)) * 2;
    auto step = [&](auto steady_tag, int it, f32x16 (&s_cur)[NQB][KB], f32x16 (&s_next)[NQB][KB]) {
      // steady state (tag true): a next tile and a tile after that exist, no branches in the main block;
      // otherwise the two conditions are evaluated at run time (the last up-to-three tiles)
      constexpr bool STEADY = decltype(steady_tag)::value;
      const bool has1 = STEADY || it + 1 < nt;
      const bool has2 = STEADY || it + 2 < nt;
      const int key0 = tile_of(it) * KT;

      // ---- mask (wave-uniform decision): ragged key tail, or a key of the tile may exceed a query of the wave;
      //      the tiles that need none come in two runs of the walk, worked out once per block
      const bool need_mask = !(it < free_a || (it >= free_b0 && it < free_b1));
      if (need_mask) {
        int qp[NQB];   // the lane's query position: derived here, where it is rarely needed, rather than kept in a register
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) qp[qb] = a.causal ? pos_of(a.qpos, min(wave_row0 + qb * 32 + l32, a.Lq - 1)) : 0;
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = key0 + kbk * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
            const bool inb = key < Lk_b;
            const int kp = a.causal ? pos_of(kpos, key) : 0;
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
              const bool vis = inb && (!a.causal || kp <= qp[qb]);
              s_cur[qb][kbk][i] = vis ? s_cur[qb][kbk][i] : -INFINITY;
            }
          }
      }

      // ---- row maxima; the running maximum only moves when a row grew by more than the threshold, so the
      //      accumulator rescale is rare (P is then bounded by 2^threshold instead of 1)
      float mc[NQB];
      bool grow = false;
      float mx[NQB];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float x = -INFINITY;
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk)
#pragma unroll
          for (int i = 0; i < 16; ++i) x = fmaxf(x, s_cur[qb][kbk][i]);
        x = both_halves_max(x);
        mx[qb] = x;
        // first visible key of a row (m_run = -inf) always takes the branch: inf > threshold
        grow = grow || ((x - m_run[qb]) * a.scale_log2 > kRescaleThreshold);
      }
      if (__any(grow)) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          const float m_new = fmaxf(m_run[qb], mx[qb]);
          const float mcn = (m_new == -INFINITY) ? 0.f : m_new * a.scale_log2;
          const float alpha = __builtin_amdgcn_exp2f(m_run[qb] * a.scale_log2 - mcn);   // m_run = -inf -> 0
          m_run[qb] = m_new;
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha;
        }
      }
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) mc[qb] = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb] * a.scale_log2;

      // ---- global prefetch: K two tiles ahead, V one tile ahead
      //      (the V tile wanted now is the K tile of the step before: its number is carried over)
      const int k_tile = tile_of(it + 2);
      if (has2) fetch(kg, k_tile, kreg);
      if (has1) fetch_v(vg, v_tile, vreg);
      v_tile = k_tile;
      // keep the loads up here: left alone, the scheduler sinks them to just before the LDS stores below to
      // save registers, and every step then waits out a full global-memory latency
      __builtin_amdgcn_sched_barrier(0);

      // ---- main block: scores of the next tile on the matrix core, softmax of this tile on the vector ALU
      if (has1) qk(kbuf + ((it + 1) & 1) * KBYTES, s_next);

      bf16x8 pf[NQB][PS];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float rs = l_run[qb];
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            u32x4 pk;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
              const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[qb][kbk][half * 8 + 2 * pr], a.scale_log2, -mc[qb]));
              const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[qb][kbk][half * 8 + 2 * pr + 1], a.scale_log2, -mc[qb]));
              f32x2 pp = {p0, p1};
              const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
              rs += p0 + p1;
              pk[pr] = __builtin_bit_cast(uint32_t, pb);
            }
            pf[qb][kbk * 2 + half] = __builtin_bit_cast(bf16x8, pk);
          }
        }
        l_run[qb] = rs;
      }

      // ---- O^T += V^T P^T   (rows = head dims, cols = queries, k = keys)
      // MFMA k index e of lane half hl in step s is key 16 s + 8 (e / 4) + 4 hl + (e % 4): the
      // accumulator layout of S^T.  The transpose read returns, for a 16-lane group whose lane j
      // points at (key base + j / 4, dim base + 4 (j % 4)), the 4 keys of dim base + j to lane j.
      const char* vlane = vbuf + (it & 1) * VBYTES + v_lane_off;
#pragma unroll
      for (int s = 0; s < PS; ++s) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          bf16x8 vf;
          if constexpr (VT) {
            // row = head dim 32 db + l32, 16 bytes = the lane half's 8 keys of k-step s in the operand's order
            vf = *(const bf16x8*)(vbuf + (it & 1) * VBYTES + (db * 32 + l32) * VSTR + 32 * s + 16 * hl);
          } else {
            const char* p0 = vlane + (16 * s) * VSTR + db * 64;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * VSTR));
            vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          }
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb)
            oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][s], oacc[qb][db], 0, 0, 0);
        }
      }

      // ---- hand the prefetched tiles to LDS: K(it+2) replaces K(it), V(it+1) replaces V(it-1)
      if (has2) stash(kbuf + (it & 1) * KBYTES, KSTR, kreg);
      if (has1) stash_v(vbuf + ((it + 1) & 1) * VBYTES, vreg);
      __syncthreads();
    };

    const std::integral_constant<bool, true> steady;
    const std::integral_constant<bool, false> draining;
    for (int blk = blk0; blk < blk1; ++blk) {
      if (per_block || MIXED) Lk_b = ap->lk_blk[blk];
      kpos = PosDesc32{ap->kpos[blk].start0, ap->kpos[blk].len0, ap->kpos[blk].start1, ap->kpos[blk].len1};
      tr = visible_key_tiles<KT>(a.causal, a.qpos, kpos, Lk_b, tile_row0, tile_row1);
      na = tr.a1 - tr.a0;
      nt = na + (tr.b1 - tr.b0);
      if (nt == 0) continue;         // nothing of this block is visible to the query tile (workgroup-uniform)
      {
        // Tiles that need no mask: full tiles that lie wholly in one ascending run of the key positions and whose
        // last key no row of this wave precedes.  In walk order they form a run at the start of each visible range.
        const int full = Lk_b / KT;
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
      vg = (const char*)ap->v[blk] + (VT ? vt_head_off : kv_head_off);

      // ---- prologue: K(0), V(0), K(1) to LDS; scores of tile 0.  (Every step ends on a barrier, so the previous
      //      block's last reads of these buffers are over.)
      full_tiles = Lk_b / KT;
      full_extent = (KT - 1) * (int)row_bytes + HS * 2;
      ragged_extent = (Lk_b - full_tiles * KT - 1) * (int)row_bytes + HS * 2;   // (not used when there is no ragged tile)
      fetch(kg, tile_of(0), kreg);
      fetch_v(vg, tile_of(0), vreg);
      stash(kbuf, KSTR, kreg);
      stash_v(vbuf, vreg);
      v_tile = tile_of(1);
      if (nt > 1) {
        fetch(kg, tile_of(1), kreg);
        stash(kbuf + KBYTES, KSTR, kreg);
      }
      __syncthreads();
      f32x16 s0[NQB][KB], s1[NQB][KB];   // scores of the current and of the next tile
      // s1 starts undefined and says so: an empty asm "defines" it.  Otherwise the compiler carries its stale value
      // from the previous block and item around every loop (the draining steps below may leave it untouched), as a
      // zero-initialised 32-register tuple that it keeps in scratch.
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int kbk = 0; kbk < KB; ++kbk) asm volatile("" : "=v"(s1[qb][kbk]));
      qk(kbuf, s0);
      __syncthreads();   // step 0 overwrites K buffer 0 with tile 2: every wave must have read tile 0 first

      int it = 0;
      for (; it + 3 < nt; it += 2) {   // two steps per trip so the score registers swap roles without copies
        step(steady, it, s0, s1);
        step(steady, it + 1, s1, s0);
      }
      for (; it < nt; ++it) {          // at most three tiles left
        step(draining, it, s0, s1);
        if (it + 1 < nt) {             // (the last step leaves s1 undefined: nothing may read it)
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
            for (int kbk = 0; kbk < KB; ++kbk) s0[qb][kbk] = s1[qb][kbk];
        }
      }
    }

    const ItemQueues queues = {ap->ticket_slot, n_items, (int)gridDim.x, ap->n_queues};
    unsigned own_ticket = kNoDraw;
    if (threadIdx.x == 0) own_ticket = queues.begin(empty_queues);
    // ---- epilogue: normalise, write O (a row that saw no key at all: l = 0 -> O = 0, LSE = -inf)
    // ---- write O (this lane: query l32, dims 32 db + 8 j + 4 hl + 0..3) and LSE
    if (STATE && !ap->state_last) {
      // not the last ring step: the state goes back as it is (each store instruction of a wave fills 1 KiB)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const f32x4 v4 = {oacc[0][db][4 * j], oacc[0][db][4 * j + 1], oacc[0][db][4 * j + 2], oacc[0][db][4 * j + 3]};
          *(f32x4*)(st_rec + ((db * 4 + j) * 64 + lane) * 4) = v4;
        }
      st_rec[DB * 16 * 64 + lane] = m_run[0];
      st_rec[DB * 16 * 64 + 64 + lane] = l_run[0];
    } else if (MIXED && per_block) {
      // a split item of a mixed launch: its partial result, fp32, dense
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float l_tot = both_halves_sum(l_run[qb]);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
        const int qrow = wave_row0 + qb * 32 + l32;
        if (qrow < a.Lq) {
          float* dst = (float*)ap->o_part[blk0] + (((size_t)b * a.Lq + qrow) * a.hq + h) * HS + 4 * hl;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const f32x4 v4 = {oacc[qb][db][4 * j] * inv, oacc[qb][db][4 * j + 1] * inv, oacc[qb][db][4 * j + 2] * inv,
                                oacc[qb][db][4 * j + 3] * inv};
              *(f32x4*)(dst + db * 32 + j * 8) = v4;
            }
          if (hl == 0)
            ap->lse_part[blk0][((size_t)b * a.hq + h) * a.Lq + qrow] = l_tot > 0.f ? m_run[qb] * a.scale + __logf(l_tot) : -INFINITY;
        }
      }
    } else
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float l_tot = both_halves_sum(l_run[qb]);
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      const int qrow = wave_row0 + qb * 32 + l32;
      if (qrow < a.Lq) {
        OutT* dst = (per_block && !MIXED) ? (OutT*)ap->o_part[blk0] + (((size_t)b * a.Lq + qrow) * a.hq + h) * HS + 4 * hl
                              : (OutT*)a.o + qo_offset(a, b, qrow, h, HS) + 4 * hl;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            f32x4 v4 = {oacc[qb][db][4 * j] * inv, oacc[qb][db][4 * j + 1] * inv, oacc[qb][db][4 * j + 2] * inv,
                        oacc[qb][db][4 * j + 3] * inv};
            OutT* d = dst + db * 32 + j * 8;
            if constexpr (sizeof(OutT) == 4) {
              *(f32x4*)d = v4;
            } else {
              u32x2 pk = {pack_bf16(v4[0], v4[1]), pack_bf16(v4[2], v4[3])};
              *(u32x2*)d = pk;
            }
          }
        if (hl == 0) {
          const float lse = l_tot > 0.f ? m_run[qb] * a.scale + __logf(l_tot) : -INFINITY;
          ((per_block && !MIXED) ? ap->lse_part[blk0] : a.lse)[((size_t)b * a.hq + h) * a.Lq + qrow] = lse;
        }
      }
    }
    if (threadIdx.x == 0) {   // waits for the draw only: the stores were issued after it
      unsigned empty = empty_queues;
      next_item[turn] = queues.finish(own_ticket, empty);
      empty_queues = empty;
    }
  }   // next work item
}

// -------------------------------------------------------------------------------------------
// fp32 instance: plain ALU, one thread per query row, key tiles staged in LDS.  Exists so that the
// ring / merge / layout logic can be checked at fp32 accuracy on fp32 inputs; not tuned.
// -------------------------------------------------------------------------------------------
template <int HS, typename OutT>
__global__ __launch_bounds__(64) void block_attn_fwd_fp32(const AttnArgs a) {
  constexpr int KT = 32;
  __shared__ float ks[KT][HS], vs[KT][HS];
  const int n_groups = a.bs * a.hkv;
  int w = blockIdx.x;
  const int group = w % n_groups; w /= n_groups;
  const int hg = w % a.g;
  const int t = w / a.g;
  const int qtile = a.causal ? a.n_qtiles - 1 - t : t;
  const int b = group / a.hkv, kvh = group % a.hkv;
  const int h = kvh * a.g + hg;
  const int row0 = qtile * 64, row1 = min(a.Lq, row0 + 64);
  const int row = row0 + threadIdx.x;
  const bool live = row < a.Lq;
  const int rr = min(row, a.Lq - 1);
  const int qp = a.causal ? pos_of(a.qpos, rr) : 0;
  const float* qsrc = (const float*)a.q + (((size_t)b * a.Lq + rr) * a.hq + h) * HS;
  float q[HS], o[HS];
#pragma unroll
  for (int e = 0; e < HS; ++e) { q[e] = qsrc[e]; o[e] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const PosDesc32 kpos = a.kpos[0];   // this instance takes one block per launch
  const TileRanges tr = visible_key_tiles<KT>(a.causal, a.qpos, kpos, a.Lk, row0, row1);
  const float* kg = (const float*)a.k[0] + ((size_t)b * a.Lk * a.hkv + kvh) * HS;
  const float* vg = (const float*)a.v[0] + ((size_t)b * a.Lk * a.hkv + kvh) * HS;
  const size_t stride = (size_t)a.hkv * HS;
  for (int pass = 0; pass < 2; ++pass) {
    const int j0 = pass ? tr.b0 : tr.a0, j1 = pass ? tr.b1 : tr.a1;
    for (int jt = j0; jt < j1; ++jt) {
      __syncthreads();
      for (int c = threadIdx.x; c < KT * HS; c += 64) {
        const int r = c / HS, e = c % HS;
        const int key = min(jt * KT + r, a.Lk - 1);
        ks[r][e] = kg[(size_t)key * stride + e];
        vs[r][e] = vg[(size_t)key * stride + e];
      }
      __syncthreads();
      for (int r = 0; r < KT; ++r) {
        const int key = jt * KT + r;
        if (key >= a.Lk) break;
        if (a.causal && pos_of(kpos, key) > qp) continue;
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < HS; ++e) s = __builtin_fmaf(q[e], ks[r][e], s);
        s *= a.scale;
        const float mn = fmaxf(m, s);
        const float alpha = expf(m - mn);     // m = -inf -> 0
        const float p = expf(s - mn);
        l = l * alpha + p;
#pragma unroll
        for (int e = 0; e < HS; ++e) o[e] = o[e] * alpha + p * vs[r][e];
        m = mn;
      }
    }
  }
  if (live) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
    OutT* dst = (OutT*)a.o + (((size_t)b * a.Lq + row) * a.hq + h) * HS;
#pragma unroll
    for (int e = 0; e < HS; ++e) dst[e] = (OutT)(o[e] * inv);
    a.lse[((size_t)b * a.hq + h) * a.Lq + row] = l > 0.f ? m + logf(l) : -INFINITY;
  }
}

template <int HS, int NQB, int NWAVES, int KT, int WPE, typename OutT, bool STATE = false, bool VT = false, bool MIXED = false>
int launch_mfma(AttnArgs a, hipStream_t stream) {
  constexpr int BM = NWAVES * NQB * 32;
  constexpr int KSTR = HS * 2 + 48, VSTR = VT ? KT * 2 + 16 : HS * 2 + 64;
  constexpr size_t lds = 2 * ((size_t)KT * KSTR + (VT ? (size_t)HS * VSTR : (size_t)KT * VSTR));
  a.n_qtiles = (a.Lq + BM - 1) / BM;
  int64_t grid = (int64_t)a.n_qtiles * a.hq * a.bs * (a.per_block ? a.n_blocks : 1);
  if constexpr (MIXED) {
    if (a.n_split_tiles < 0 || a.n_split_tiles > a.n_qtiles) return USP_ERR_UNSUPPORTED;
    const int64_t split = (int64_t)a.n_split_tiles * a.hq * a.bs * a.n_blocks;
    grid = split + (int64_t)(a.n_qtiles - a.n_split_tiles) * a.hq * a.bs;
    if (split > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
    a.n_split_items = (int)split;
  }
  if (grid > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
  auto kern = block_attn_fwd_mfma<HS, NQB, NWAVES, KT, WPE, OutT, STATE, VT, MIXED>;
  static LdsLimitRaised lds_limit;   // per kernel instance
  if (!raise_dynamic_lds_limit((const void*)kern, lds, lds_limit)) return USP_ERR_LAUNCH;
  // one workgroup per CU (its registers and LDS fill a CU), fewer when there are fewer items
  a.ticket_slot = ticket_slot_for(stream);
  a.n_items = (int)grid;
  a.n_queues = std::gcd(dev::kMaxItemQueues, a.bs * a.hkv);
  const int n_wgs = (int)std::min<int64_t>(grid, compute_units());
  hipLaunchKernelGGL(kern, dim3((unsigned)n_wgs), dim3(NWAVES * 64), lds, stream, a);
  return launch_status();
}

template <int HS, typename OutT>
int launch_fp32(AttnArgs a, hipStream_t stream) {
  a.n_qtiles = (a.Lq + 63) / 64;
  const int64_t grid = (int64_t)a.n_qtiles * a.hq * a.bs;
  if (grid > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((block_attn_fwd_fp32<HS, OutT>), dim3((unsigned)grid), dim3(64), 0, stream, a);
  return launch_status();
}

}  // namespace

int launch_ring_attn_fwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                         int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc& qpos,
                         int in_dtype, int o_dtype, hipStream_t stream, const SeqLayoutIO* seq, const RingState* state,
                         bool v_transposed) {
  if (n_blocks < 1 || n_blocks > kMaxBlocks) return USP_ERR_UNSUPPORTED;
  if (in_dtype == USP_FP32 && (n_blocks != 1 || seq)) return USP_ERR_UNSUPPORTED;
  AttnArgs a;
  a.seq_n = seq ? seq->rows_per_shard : 0;
  a.seq_heads = seq ? seq->heads : 0;
  a.seq_head0 = seq ? seq->head0 : 0;
  a.q = q; a.o = o; a.lse = lse;
  for (int j = 0; j < kMaxBlocks; ++j) {
    const int jj = j < n_blocks ? j : 0;
    a.k[j] = k_blocks[jj];
    a.v[j] = v_blocks[jj];
    const usp_posdesc& kp = kpos_blocks[jj];
    a.kpos[j] = PosDesc32{(int)kp.start0, (int)kp.len0, (int)kp.start1, (int)kp.len1};
  }
  a.n_blocks = n_blocks;
  a.per_block = 0;
  a.n_split_items = a.n_split_tiles = 0;
  a.state = state ? state->state : nullptr;
  a.state_first = state ? state->first : 0;
  a.state_last = state ? state->last : 0;
  if (state && in_dtype != USP_BF16) return USP_ERR_DTYPE;
  for (int j = 0; j < kMaxBlocks; ++j) {
    a.lk_blk[j] = (int)Lk;
    a.o_part[j] = nullptr;
    a.lse_part[j] = nullptr;
  }
  a.bs = bs; a.hq = hq; a.hkv = hkv; a.g = hq / hkv;
  a.Lq = (int)Lq; a.Lk = (int)Lk;
  a.n_qtiles = 0;
  a.ticket_slot = 0;
  a.n_items = 0;
  a.n_queues = 1;
  a.causal = causal;
  a.scale = scale;
  a.scale_log2 = scale * 1.4426950408889634f;
  a.qpos = PosDesc32{(int)qpos.start0, (int)qpos.len0, (int)qpos.start1, (int)qpos.len1};
  if (in_dtype == USP_FP32) {
    if (hs == 128) return o_dtype == USP_FP32 ? launch_fp32<128, float>(a, stream) : launch_fp32<128, __bf16>(a, stream);
    return o_dtype == USP_FP32 ? launch_fp32<64, float>(a, stream) : launch_fp32<64, __bf16>(a, stream);
  }
  if (state && v_transposed) return USP_ERR_UNSUPPORTED;
  if (v_transposed) {   // V blocks in key-tile-transposed layout (bf16 in and out)
    if (in_dtype != USP_BF16 || o_dtype != USP_BF16) return USP_ERR_DTYPE;
    return hs == 128 ? launch_mfma<128, 1, 8, 64, 2, __bf16, false, true>(a, stream)
                     : launch_mfma<64, 1, 8, 64, 2, __bf16, false, true>(a, stream);
  }
  if (a.state) {   // the instance that reads and writes the running state of a step-by-step ring
    if (hs == 128)
      return o_dtype == USP_FP32 ? launch_mfma<128, 1, 8, 64, 2, float, true>(a, stream)
                                 : launch_mfma<128, 1, 8, 64, 2, __bf16, true>(a, stream);
    return o_dtype == USP_FP32 ? launch_mfma<64, 1, 8, 64, 2, float, true>(a, stream)
                               : launch_mfma<64, 1, 8, 64, 2, __bf16, true>(a, stream);
  }
  // 256 query rows per workgroup (8 waves x 32), 64-key tiles, two waves per SIMD
  if (hs == 128)
    return o_dtype == USP_FP32 ? launch_mfma<128, 1, 8, 64, 2, float>(a, stream)
                               : launch_mfma<128, 1, 8, 64, 2, __bf16>(a, stream);
  if (o_dtype == USP_FP32) return launch_mfma<64, 1, 8, 64, 2, float>(a, stream);
  return launch_mfma<64, 1, 8, 64, 2, __bf16>(a, stream);
}

int launch_block_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int bs, int64_t Lq,
                          int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc& qpos,
                          const usp_posdesc& kpos, int in_dtype, int o_dtype, hipStream_t stream) {
  return launch_ring_attn_fwd(q, &k, &v, &kpos, 1, o, lse, bs, Lq, Lk, hq, hkv, hs, scale, causal, qpos, in_dtype,
                              o_dtype, stream);
}

size_t attn_fwd_state_bytes(int bs, int64_t Lq, int hq, int hs) {
  // one record per 32-row block, query tiles of 256 rows rounded up (the kernel's item shape)
  return (size_t)bs * hq * (size_t)((Lq + 255) / 256) * 8 * state_record_floats(hs) * sizeof(float);
}

int launch_attn_fwd_partials(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                             const usp_posdesc* kpos_blocks, const int* lk_blocks, int n_blocks, float* const* o_parts,
                             float* const* lse_parts, int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                             float scale, int causal, const usp_posdesc& qpos, hipStream_t stream,
                             const SeqLayoutIO* seq, const MixedLaunch* mixed) {
  if (n_blocks < 1 || n_blocks > kMaxBlocks) return USP_ERR_UNSUPPORTED;
  if (mixed && mixed->v_transposed)   // a piece of transposed tiles begins with a whole tile, 16-byte aligned
    for (int j = 0; j < n_blocks; ++j)
      if ((uintptr_t)v_blocks[j] & 15) return USP_ERR_UNSUPPORTED;
  AttnArgs a;
  a.seq_n = seq ? seq->rows_per_shard : 0;
  a.seq_heads = seq ? seq->heads : 0;
  a.seq_head0 = seq ? seq->head0 : 0;
  a.q = q; a.o = nullptr; a.lse = nullptr;
  for (int j = 0; j < kMaxBlocks; ++j) {
    const int jj = j < n_blocks ? j : 0;
    a.k[j] = k_blocks[jj];
    a.v[j] = v_blocks[jj];
    const usp_posdesc& kp = kpos_blocks[jj];
    a.kpos[j] = PosDesc32{(int)kp.start0, (int)kp.len0, (int)kp.start1, (int)kp.len1};
    a.lk_blk[j] = lk_blocks ? lk_blocks[jj] : (int)Lk;
    if (a.lk_blk[j] < 1 || a.lk_blk[j] > Lk) return USP_ERR_SHAPE;
    a.o_part[j] = o_parts[jj];
    a.lse_part[j] = lse_parts[jj];
  }
  a.n_blocks = n_blocks;
  a.per_block = 1;
  a.n_split_items = a.n_split_tiles = 0;
  a.state = nullptr;
  a.state_first = a.state_last = 0;
  a.bs = bs; a.hq = hq; a.hkv = hkv; a.g = hq / hkv;
  a.Lq = (int)Lq; a.Lk = (int)Lk;
  a.n_qtiles = 0;
  a.ticket_slot = 0;
  a.n_items = 0;
  a.n_queues = 1;
  a.causal = causal;
  a.scale = scale;
  a.scale_log2 = scale * 1.4426950408889634f;
  a.qpos = PosDesc32{(int)qpos.start0, (int)qpos.len0, (int)qpos.start1, (int)qpos.len1};
  if (mixed) {
    a.o = mixed->o;
    a.lse = mixed->lse;
    a.per_block = 0;
    a.n_split_tiles = mixed->n_split_tiles;
    if (mixed->v_transposed)
      return hs == 128 ? launch_mfma<128, 1, 8, 64, 2, __bf16, false, true, true>(a, stream)
                       : launch_mfma<64, 1, 8, 64, 2, __bf16, false, true, true>(a, stream);
    return hs == 128 ? launch_mfma<128, 1, 8, 64, 2, __bf16, false, false, true>(a, stream)
                     : launch_mfma<64, 1, 8, 64, 2, __bf16, false, false, true>(a, stream);
  }
  return hs == 128 ? launch_mfma<128, 1, 8, 64, 2, float>(a, stream) : launch_mfma<64, 1, 8, 64, 2, float>(a, stream);
}

}  // namespace usp
