/* usp.h -- C ABI of the MI355X (gfx950) USP attention library.
 *
 * USP = unified Ulysses x Ring sequence-parallel attention (arxiv 2405.07719, Sec. 3,
 * Algorithm 1).  This library runs one rank's share of that path on ONE GPU; the other
 * ranks of the SP group are "virtual": their shards live in the same device buffers,
 * the Ulysses all-to-all is a local permutation and the ring is a loop over resident
 * K/V blocks.  No inter-GPU communication happens here.
 *
 * Conventions for every entry point
 *   - returns a usp_status (0 = USP_OK); never throws, aborts or synchronises;
 *   - all tensor pointers are DEVICE pointers owned by the caller, dense, row-major in
 *     the stated shape; the library keeps no reference after return;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream);
 *   - arguments are validated on the host BEFORE any launch; on error nothing is enqueued;
 *   - no device memory is allocated: scratch comes from the caller (`workspace`), its
 *     size from the matching *_workspace_bytes query (host only, works without a GPU);
 *   - calls may be issued from several host threads and on several streams.  The bf16 attention kernels (forward,
 *     dQ, dK/dV) hand out their work through sets of counters in static device arrays (256 KiB per kernel file), each
 *     set back at zero when its launch ends.  Every stream gets a set of its own (launches on one stream never
 *     overlap), and so does every graph capture: calls on different streams, and graph replays beside eager calls,
 *     cannot meet in a set.  What remains: two executable graphs instantiated from ONE capture must not be replayed
 *     at the same time; and a process that has used more than 3840 distinct streams and captures shares the last 256
 *     sets in rotation among the later ones.
 *
 * Notation (Sec. 2, notation table): L sequence length, hc head count, hs head size,
 * bs batch.  Added: hk = KV head count (GQA), U = Ulysses degree, R = ring degree,
 * N = U*R (Sec. 3), Lq = L/R, hq = hc/U, hkv = hk/U.
 * Virtual rank numbering: rank = r*U + u, Ulysses fastest (Sec. 4, Tip 7 ordering).
 *
 * Buffer layouts
 *   seq layout  : [N][bs][L/N][heads][hs]     one input/output shard per rank (Sec. 3)
 *   head layout : [N][bs][L/R][heads/U][hs]   after the forward all-to-all
 *   lse         : [N][bs][hc/U][L/R] float    rank-local head layout (Algorithm 1
 *                                             all-to-alls only O back)
 */
#ifndef USP_H_
#define USP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(USP_BUILDING)
#pragma GCC visibility push(default)
#endif

typedef enum {
  USP_OK = 0,
  USP_ERR_NULL = 1,        /* a required pointer is NULL */
  USP_ERR_SHAPE = 2,       /* non-positive size; L not divisible by N (contiguous) or 2*R*U (zigzag) */
  USP_ERR_DEGREE = 3,      /* U<1, R<1, hc%U, hk%U (Ulysses degree cannot exceed/divide the KV heads, Sec. 3), hc%hk */
  USP_ERR_DTYPE = 4,       /* unknown or unsupported dtype combination */
  USP_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than the query says */
  USP_ERR_UNSUPPORTED = 6, /* e.g. hs not in {64,128}, too many merge parts, rank range out of bounds */
  USP_ERR_LAUNCH = 7       /* the HIP runtime reported an error when enqueuing */
} usp_status;

typedef enum { USP_BF16 = 0, USP_FP32 = 1 } usp_dtype;
typedef enum { USP_SPLIT_CONTIG = 0, USP_SPLIT_ZIGZAG = 1 } usp_split; /* basic ring vs load-balanced ring (Sec. 3) */
/* forward / reverse AllToAll4D (Algorithm 1); USP_SEQ_TO_HEAD_VT: the forward one with the head-layout side in the
 * key-tile-transposed layout that usp_ring_attn_fwd_vt reads (see usp_layout_a2a) */
typedef enum { USP_SEQ_TO_HEAD = 0, USP_HEAD_TO_SEQ = 1, USP_SEQ_TO_HEAD_VT = 2 } usp_a2a_dir;

/* The problem of Algorithm 1.  scale = 0 means 1/sqrt(hs) (Eq. 1 read per head). */
typedef struct {
  int32_t bs;
  int64_t L;
  int32_t hc, hk, hs;
  int32_t ulysses, ring;
  int32_t causal;   /* 0 / 1 */
  int32_t split;    /* usp_split: how ring blocks are cut from the sequence */
  int32_t dtype;    /* usp_dtype of Q, K, V, O (and dO, dQ, dK, dV) */
  float scale;
} usp_problem;

/* Global positions of a local index range in at most two ascending runs (Algorithm 2 gives
 * two chunks per ring rank): local i < len0 -> start0 + i, otherwise start1 + (i - len0). */
typedef struct {
  int64_t start0, len0, start1, len1;
} usp_posdesc;

#define USP_MAX_MERGE_PARTS 64
#define USP_MAX_RING_BLOCKS 16

/* Text for a status code (static storage). */
const char* usp_status_str(int status);

/* Host only.  Checks a problem against the constraints of Sec. 3 (degrees vs head counts,
 * divisibility of L).  Returns USP_OK or the first violated class. */
int usp_validate(const usp_problem* p);

/* Host only.  Algorithm 2 as index arithmetic for virtual rank (ring_rank, ulysses_rank):
 *   *shard      <- positions of its [L/N] input shard (the u-th of U pieces of the ring block);
 *   *ring_block <- positions of ring rank r's [L/R] block (zigzag: chunks r and 2R-1-r of 2R;
 *                  contiguous: block r of R).
 * Either output pointer may be NULL. */
int usp_local_positions(const usp_problem* p, int ring_rank, int ulysses_rank, usp_posdesc* shard,
                        usp_posdesc* ring_block);

/* Algorithm 1 steps 2-4 (dir = USP_SEQ_TO_HEAD) and 6 (USP_HEAD_TO_SEQ): the AllToAll4D of one
 * Ulysses group as a permutation.  `heads` is hc (Q, O) or hk (K, V); element size from p->dtype.
 * Ranks [rank_begin, rank_end) index the HEAD-layout side:
 *   SEQ_TO_HEAD: for each such rank (r,u) gather   dst_head[rank][b][u'*(L/N)+s][h'][e] =
 *                src_seq[r*U+u'][b][s][u*(heads/U)+h'][e]   for all u' in [0,U);
 *   HEAD_TO_SEQ: for each such rank scatter the inverse (it fills its head slice of the U
 *                seq-layout shards of its Ulysses group).
 *   SEQ_TO_HEAD_VT: the same gather (bf16 data only) with each rank's head-layout block transposed in tiles of 64
 *                rows: dst[rank] = [bs][heads/U][ceil((L/R)/64)][hs][64], place j of tile t holding the element of
 *                local row 64 t + 16 (j/16) + order[j%16], order = 0,1,2,3, 8,9,10,11, 4,5,6,7, 12,13,14,15 (the
 *                order in which the matrix instruction's operand holds 16 keys); places past the last row are
 *                zeros; a rank's block takes bs * heads/U * ceil((L/R)/64) * 64 * hs * 2 bytes.  For V: the
 *                attention kernel then reads its V operand with plain 16-byte reads (usp_ring_attn_fwd_vt).
 * src and dst are whole-buffer base pointers (seq or head layout as the direction implies)
 * and must not overlap.  Bit-exact copy; no arithmetic. */
int usp_layout_a2a(const usp_problem* p, int heads, int dir, const void* src, void* dst, int rank_begin,
                   int rank_end, void* stream);

/* One ring step (Sec. 2, the blockwise loop of SP-Ring; Eq. 1 restricted to one K/V block).
 *   q [bs,Lq,hq,hs]; k, v [bs,Lk,hkv,hs]  (in_dtype);  query head h reads KV head h / (hq/hkv);
 *   o_part [bs,Lq,hq,hs] (o_dtype): softmax(scale*q k^T) v over the VISIBLE keys of this block;
 *   lse_part [bs,hq,Lq] float: natural-log sum of exp(scale*q.k) over the visible keys.
 * causal != 0: key j is visible to query i iff kpos(j) <= qpos(i) (global positions from the
 * descriptors); causal == 0: every key is visible and qpos/kpos may be NULL.
 * A row with no visible key gets o = 0 and lse = -inf.  scale = 0 means 1/sqrt(hs).
 * bf16 inputs run on MFMA with fp32 accumulation; fp32 inputs run a plain-ALU instance. */
int usp_block_attn_fwd(const void* q, const void* k, const void* v, void* o_part, float* lse_part, int bs,
                       int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                       const usp_posdesc* qpos, const usp_posdesc* kpos, int in_dtype, int o_dtype,
                       void* stream);

/* One ring step with the running state carried from call to call (Sec. 2: the blockwise loop of SP-Ring keeps, per
 * query row, the running maximum, the running sum and the unnormalised output, and folds one K/V block after the
 * other into them): for a ring that RECEIVES its blocks one per step there are no partial outputs to keep and no
 * merge pass.  Call it once per arriving block, in any order of the blocks, with the same q, qpos and state:
 *   first != 0: the state is started (not read);  otherwise it is read and continued;
 *   last  != 0: the final o [bs,Lq,hq,hs] (o_dtype) and lse [bs,hq,Lq] float are written (normalised, natural-log
 *               LSE; a row that saw no key in any step gets o = 0, lse = -inf) and the state is left as it was;
 *               otherwise the state is written back and o, lse are not touched (they may be NULL).
 * The result after the last call equals usp_block_attn_fwd per block + usp_lse_merge, and usp_ring_attn_fwd over
 * all blocks, up to rounding.  state: DEVICE memory of usp_block_attn_fwd_state_bytes() bytes, 16-byte aligned, in
 * a layout private to the library (registers of the kernel, as they are); valid only between calls of the same
 * shape.  bf16 inputs; everything else as in usp_block_attn_fwd. */
size_t usp_block_attn_fwd_state_bytes(int bs, int64_t Lq, int hq, int hs);
int usp_block_attn_fwd_state(const void* q, const void* k, const void* v, void* state, size_t state_bytes, void* o,
                             float* lse, int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale,
                             int causal, const usp_posdesc* qpos, const usp_posdesc* kpos, int first, int last,
                             int o_dtype, void* stream);

/* Merge of the ring steps' partial results (implied by the blockwise formulation of Sec. 2):
 *   lse_out = ln sum_i exp(lse_i);  o_out = sum_i exp(lse_i - lse_out) * o_i;
 * parts with lse_i = -inf contribute nothing; all -inf gives (0, -inf).
 * o_parts / lse_parts: HOST arrays of n_parts DEVICE pointers, each [bs,Lq,hq,hs] (part_dtype)
 * and [bs,hq,Lq] float; 1 <= n_parts <= USP_MAX_MERGE_PARTS.  hs must be a multiple of 8.
 * Aliasing: o_out may be the very buffer of one part (same address) when part_dtype == out_dtype and hs is 64 or
 * 128 (every thread then overwrites exactly the bytes it has read, and the threads of a row share a wavefront), and
 * lse_out may then be that part's lse buffer; any other overlap of an output with a part is rejected
 * (USP_ERR_UNSUPPORTED). */
int usp_lse_merge(const void* const* o_parts, const float* const* lse_parts, int n_parts, void* o_out,
                  float* lse_out, int bs, int64_t Lq, int hq, int hs, int part_dtype, int out_dtype,
                  void* stream);

/* The whole ring loop of one rank in ONE launch (Algorithm 1 step 5 with the merge folded in; Sec. 2, the
 * blockwise loop of SP-Ring): attention of q over the n_blocks K/V blocks that are already resident, each of
 * Lk keys with its own position descriptor.  The online-softmax state of a query row (running maximum, sum and
 * unnormalised output) stays in registers from the first block to the last, so there are no partial outputs and
 * no merge pass; the result equals usp_block_attn_fwd per block followed by usp_lse_merge, up to rounding.
 *   k_blocks, v_blocks: HOST arrays of n_blocks DEVICE pointers, each [bs,Lk,hkv,hs]; kpos_blocks: HOST array
 *   of n_blocks descriptors (ignored, may be NULL, when causal == 0); 1 <= n_blocks <= USP_MAX_RING_BLOCKS;
 *   bf16 inputs only (in_dtype is checked); o [bs,Lq,hq,hs] (o_dtype), lse [bs,hq,Lq] float.
 * Everything else as in usp_block_attn_fwd.  The order of the blocks changes the result only by rounding. */
int usp_ring_attn_fwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                      const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                      int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                      int in_dtype, int o_dtype, void* stream);

/* usp_ring_attn_fwd with the V blocks in the key-tile-transposed layout of USP_SEQ_TO_HEAD_VT (each block
 * [bs][hkv][ceil(Lk/64)][hs][64], 16-byte aligned; K blocks as before): the transposition of V that the P V product
 * needs has then been done once, by the permutation that Algorithm 1's all-to-all is anyway, instead of at every
 * read of a tile (a third fewer LDS reads per step; 3 % faster).  bf16 in and out; same results as
 * usp_ring_attn_fwd bit for bit.  usp_attn_fwd uses it internally. */
int usp_ring_attn_fwd_vt(const void* q, const void* const* k_blocks, const void* const* vt_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                         int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc* qpos,
                         void* stream);

/* The same query rows against n_blocks K/V blocks with the key dimension SPLIT over the chip (Sec. 2: the
 * blockwise loop gives partial results that combine by their log-sum-exp, in any grouping): every (query tile,
 * head, batch, block) is its own work item of ONE launch, and block j's result goes to its own partial,
 * o_parts[j] [bs,Lq,hq,hs] fp32 and lse_parts[j] [bs,hq,Lq] float, for usp_lse_merge to combine.  For short
 * sequences, where the rows of the last query tile alone (one workgroup per tile and head) would take longer
 * than the whole chip needs for everything: the blocks may be pieces of one K/V tensor.
 *   k_blocks, v_blocks: HOST arrays of n_blocks DEVICE pointers to the first row of each block; rows are hkv*hs
 *   elements apart, batches Lk rows apart (so pieces of a [bs,Lk,hkv,hs] tensor are blocks of it);
 *   lk_blocks: HOST array, keys in each block, 1 <= lk_blocks[j] <= Lk (NULL: Lk each); kpos_blocks as in
 *   usp_ring_attn_fwd, describing lk_blocks[j] keys each; o_parts, lse_parts: HOST arrays of DEVICE pointers;
 *   bf16 inputs.  A query row that sees no key of block j gets o = 0, lse = -inf there. */
int usp_ring_attn_fwd_partials(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                               const usp_posdesc* kpos_blocks, const int32_t* lk_blocks, int n_blocks,
                               float* const* o_parts, float* const* lse_parts, int bs, int64_t Lq, int64_t Lk, int hq,
                               int hkv, int hs, float scale, int causal, const usp_posdesc* qpos, void* stream);

/* Algorithm 1 forward for virtual ranks [rank_begin, rank_end):
 * all-to-all of Q,K,V -> ring loop of block attention -> LSE merge -> all-to-all of O.
 * With bf16 data and R <= USP_MAX_RING_BLOCKS the ring loop and the merge are the single launch of
 * usp_ring_attn_fwd (all blocks are resident on the one GPU); otherwise one usp_block_attn_fwd per ring step
 * with fp32 partials, then usp_lse_merge.  Short sequences (fewer query tiles x heads than keep 256 CUs busy for
 * as long as the last tile takes) run the single launch of usp_ring_attn_fwd_partials over two to eight parts of
 * the keys, then usp_lse_merge; a little longer (more than one work item per CU, the heaviest still longer than
 * a CU's share) only the last query tiles of a causal rank are cut so, in the same launch as the whole ones, and
 * the merge covers their rows; the workspace query knows.
 *   q, o: seq layout with hc heads; k, v: seq layout with hk heads (ALL N shards must be
 *   present: the ring reads the other ring ranks' K/V where hardware would receive them);
 *   lse: [N][bs][hc/U][L/R] float, written for the ranks in range.
 * With Ulysses degree 1 the all-to-alls are the identity (a block in head layout is its shard as it stands): K, and
 * V unless re-tiling it pays, are read where the caller holds them, not copied.
 * The workspace query returns 0 for an invalid problem or n_ranks < 1, and also for a plan that needs none (a
 * ring-only bf16 problem whose ring loop is one launch): usp_attn_fwd then accepts any workspace pointer, NULL
 * included; usp_validate tells the two apart. */
size_t usp_attn_fwd_workspace_bytes(const usp_problem* p, int n_ranks);
int usp_attn_fwd(const usp_problem* p, const void* q, const void* k, const void* v, void* o, float* lse,
                 int rank_begin, int rank_end, void* workspace, size_t workspace_bytes, void* stream);

/* usp_attn_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same
 * kernels, same results bit for bit (with one exception: where usp_attn_fwd would cut a rank's heaviest query tiles
 * and the partial results of that cut do not fit the array, the launch stays whole: same attention, another rounding
 * order).  The scratch is a static device array of USP_NOALLOC_SCRATCH_BYTES that every
 * GPU the library runs on holds until the process ends; the call allocates and frees nothing.  A problem whose
 * usp_attn_fwd workspace (for the Ulysses columns the rank range touches; without those optional partials) is
 * larger returns USP_ERR_WORKSPACE and
 * enqueues nothing: one rank of L = 212992, U 8 x R 2 (104 MiB) fits, a whole 16-rank range of it does not.  All
 * calls on one GPU share the one array: calls that overlap in time on one GPU (different streams) race; calls on
 * one stream are safe.  The array keeps the last call's contents; every region is rewritten before it is read. */
#define USP_NOALLOC_SCRATCH_BYTES ((size_t)128 << 20)
int usp_attn_fwd_noalloc(const usp_problem* p, const void* q, const void* k, const void* v, void* o, float* lse,
                         int rank_begin, int rank_end, void* stream);

/* D_i = sum_e dO[i][e] * O[i][e] per (batch, position, head) row: the row term of the softmax gradient
 * (textbook backward of Eq. 1).  o, d_o [bs,L,h,hs] bf16 -> delta [bs,h,L] float. */
int usp_attn_delta(const void* o, const void* d_o, float* delta, int bs, int64_t L, int h, int hs, void* stream);

/* Backward of one ring step (gradient of Eq. 1 restricted to one K/V block; shapes and mask as in
 * usp_block_attn_fwd; bf16 inputs only).  lse [bs,hq,Lq] is the FINAL log-sum-exp of each query row over
 * all blocks (as usp_attn_fwd / usp_lse_merge return it) and delta comes from usp_attn_delta, so that
 * P_ij = exp(scale q_i.k_j - lse_i) is exact and contributions of different blocks add:
 *   dq [bs,Lq,hq,hs]  (+)= scale * sum_j dS_ij k_j      dS_ij = P_ij (dO_i.v_j - delta_i)
 *   dk [bs,Lk,hkv,hs] (+)= scale * sum_i dS_ij q_i      (summed over the query heads of the KV head's group)
 *   dv [bs,Lk,hkv,hs] (+)= sum_i P_ij dO_i
 * dq, dk, dv are fp32; accumulate = 0 overwrites them, 1 adds to them.  dq is deterministic; dk and dv are
 * summed over the query heads of a group either inside one workgroup (large grids) or by fp32 atomic adds of at
 * most hq/hkv addends per element (small grids), whose rounding depends on their order. */
int usp_block_attn_bwd(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                       const float* delta, float* dq, float* dk, float* dv, int bs, int64_t Lq, int64_t Lk, int hq,
                       int hkv, int hs, float scale, int causal, const usp_posdesc* qpos, const usp_posdesc* kpos,
                       int accumulate, void* stream);

/* Backward of a rank's whole ring loop over its n_blocks resident K/V blocks in one launch pair (the backward
 * counterpart of usp_ring_attn_fwd; same result as one usp_block_attn_bwd per block, up to rounding).
 *   k_blocks, v_blocks, dk_blocks, dv_blocks: HOST arrays of n_blocks DEVICE pointers ([bs,Lk,hkv,hs]; bf16 inputs,
 *   fp32 gradients); kpos_blocks: HOST array of n_blocks descriptors (may be NULL when causal == 0);
 *   accumulate_dq: 0 overwrites dq, 1 adds; accumulate_dkdv: HOST array of n_blocks flags, per block.
 *   1 <= n_blocks <= USP_MAX_RING_BLOCKS; the blocks' gradient buffers must not overlap. */
int usp_ring_attn_bwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                      const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                      const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks, int bs,
                      int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                      const usp_posdesc* qpos, int accumulate_dq, const int* accumulate_dkdv, void* stream);

/* usp_ring_attn_bwd with a workspace (same arguments, same results up to rounding): problems whose work items
 * are few and long (short sequences) or whose query heads are split over workgroups are cut into slices that
 * each write their own fp32 copy of dq / dk / dv into the workspace, and one more pass adds the copies up into
 * the outputs (adding to what is there where the accumulate flags say so).  No atomic adds: the results do not
 * depend on the order in which workgroups finish, and on such problems it is the faster of the two.  The
 * workspace size is a function of the shape alone (0: no copies needed, the call is usp_ring_attn_bwd).
 * With at least usp_ring_attn_bwd_workspace_bytes_with_ds() bytes (2 bytes more per (query, key) pair of the call,
 * lengths rounded up to 256) the dK/dV kernel keeps its dS for the dQ kernel, as described at usp_attn_bwd. */
size_t usp_ring_attn_bwd_workspace_bytes(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs, int n_blocks);
size_t usp_ring_attn_bwd_workspace_bytes_with_ds(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                                                 int n_blocks);
int usp_ring_attn_bwd_ws(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                         const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks, int bs,
                         int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                         const usp_posdesc* qpos, int accumulate_dq, const int* accumulate_dkdv, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Algorithm 1 backward (Sec. 3: the all-to-alls swap their scatter/gather roles) for virtual ranks
 * [rank_begin, rank_end); bf16 problems only.
 *   q, k, v, o, d_o: seq layout (o as usp_attn_fwd wrote it); lse: [N][bs][hc/U][L/R] from usp_attn_fwd;
 *   dq, dk, dv: seq layout outputs in the problem dtype.
 * Per rank: all-to-all of Q and dO -> delta (O and dO read at their places in the shards) -> R block backwards (dQ
 * accumulated over the ring steps in fp32; the dK/dV contribution of step i is added to block (r-i) mod R's fp32
 * accumulator, the buffer that would travel the ring with the block) -> dQ converted and scattered back to the
 * shards.  After the last rank the dK/dV accumulators are converted and scattered back likewise.
 * dq is complete for the ranks in range (each fills its head slice of its Ulysses group's shards).
 * dk/dv: for every Ulysses column u that has a rank (r,u) in range, the column's head slice of ALL N shards is
 * OVERWRITTEN with the sum of the contributions of the column's ranks in range; the head slices of columns
 * without a rank in range are not written.  Complete dk/dv therefore needs rank_begin = 0, rank_end = N (or
 * all R ring rows of one column for that column's head slice).
 * The fp32 accumulators may be held in several copies (one per slice of the work that a short or narrow problem is
 * cut into, each written with plain stores and added up by the conversion pass; the workspace query knows): the
 * results do not depend on the order in which workgroups finish.
 * Optional, for callers with memory to spare: a workspace of at least usp_attn_bwd_workspace_bytes_with_ds() bytes
 * (the plain size plus 2 bytes per (query, key) pair, masked or not, of one rank's ring loop: bs * hc/U * R *
 * (L/R)^2 * 2, keys and queries rounded up to 256) lets the dK/dV kernel keep the dS it forms, as bf16, and
 * the dQ kernel read it back instead of forming S and dP a second time: 5 matrix products per tile pair instead
 * of 7.  Same results up to the bf16 rounding of dS, which both kernels apply anyway.  Chosen by workspace_bytes
 * alone; any size from usp_attn_bwd_workspace_bytes() up is accepted.  Head size 128 only: at head size 64 the second
 * pair of products costs less than moving dS, the _with_ds query returns the plain size and more room is ignored. */
size_t usp_attn_bwd_workspace_bytes(const usp_problem* p, int n_ranks);
size_t usp_attn_bwd_workspace_bytes_with_ds(const usp_problem* p, int n_ranks);
int usp_attn_bwd(const usp_problem* p, const void* q, const void* k, const void* v, const void* o,
                 const float* lse, const void* d_o, void* dq, void* dk, void* dv, int rank_begin,
                 int rank_end, void* workspace, size_t workspace_bytes, void* stream);

#if defined(USP_BUILDING)
#pragma GCC visibility pop
#endif

#ifdef __cplusplus
}
#endif
#endif /* USP_H_ */
