// Internal declarations shared by the translation units of libusp.so (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "usp.h"

namespace usp {

// CUs of the chip the work-splitting plans are made for (MI355X).  The plans (key splits of the forward, slices and
// head splits of the backward) size workspaces, and the workspace queries must work without a GPU, so this is a
// constant and the ONE place it is written; the launchers ask the device for its CU count only to size their grids
// (a plan made for another CU count is still correct, only less well balanced).
constexpr int kPlanCUs = 256;

inline size_t dtype_size(int dt) { return dt == USP_BF16 ? 2 : (dt == USP_FP32 ? 4 : 0); }

// Global position of local index i under a two-run descriptor.
__host__ __device__ inline int64_t pos_of(const usp_posdesc& d, int64_t i) {
  return i < d.len0 ? d.start0 + i : d.start1 + (i - d.len0);
}

// Smallest / largest global position over local indices [a, b), b > a, within the descriptor.
__host__ __device__ inline int64_t pos_min(const usp_posdesc& d, int64_t a, int64_t b) {
  int64_t m = INT64_MAX;
  if (a < d.len0) m = d.start0 + a;
  if (b > d.len0) {
    int64_t a1 = (a > d.len0 ? a : d.len0) - d.len0;
    int64_t v = d.start1 + a1;
    m = v < m ? v : m;
  }
  return m;
}
__host__ __device__ inline int64_t pos_max(const usp_posdesc& d, int64_t a, int64_t b) {
  int64_t m = INT64_MIN;
  if (a < d.len0) {
    int64_t e = b < d.len0 ? b : d.len0;
    m = d.start0 + e - 1;
  }
  if (b > d.len0) {
    int64_t v = d.start1 + (b - 1 - d.len0);
    m = v > m ? v : m;
  }
  return m;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? USP_OK : USP_ERR_LAUNCH; }

// Raises a kernel's limit of dynamic LDS, once per kernel instance and device (the attribute belongs to the device's
// copy of the function).  `done` is the instance's own record, a function-local static of the caller; later calls,
// which may come during stream capture, only read it.  Two threads that meet here both set the same value.
struct LdsLimitRaised { std::atomic<bool> on_device[64]; };
inline bool raise_dynamic_lds_limit(const void* kernel, size_t bytes, LdsLimitRaised& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  if (done.on_device[dev].load(std::memory_order_acquire)) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
  done.on_device[dev].store(true, std::memory_order_release);
  return true;
}

// Kernel launchers (defined next to their kernels).  All take validated arguments.
// Ranks rank_begin, rank_begin + rank_step, ... below rank_end are transformed in one launch.
// head_rank_base >= 0: the rank whose slot the head-layout base pointer points at (0 for a whole buffer);
// head_rank_base < 0: the head-layout side is a packed workspace holding the launch's ranks back to back.
int launch_layout_a2a(const usp_problem& p, int heads, int dir, const void* src, void* dst, int rank_begin,
                      int rank_end, int head_rank_base, hipStream_t stream, int rank_step = 1);
// The same for up to USP_LAYOUT_MAX_TENSORS tensors of one geometry (same heads, ranks and head_rank_base) in ONE launch.
#define USP_LAYOUT_MAX_TENSORS 3
int launch_layout_a2a_multi(const usp_problem& p, int heads, int dir, int n_tensors, const void* const* src,
                            void* const* dst, int rank_begin, int rank_end, int head_rank_base, hipStream_t stream,
                            int rank_step = 1);
// Optional: Q is read from and O written to the sequence-layout shards of the rank's Ulysses group
// ([U][bs][rows_per_shard][heads][hs], q and o pointing at the group's first shard) instead of dense head-layout
// tensors; head0 is the rank's first head.  Attention kernels: bf16 instance only.  Merge: fp32 partials only (the
// merged O goes to the shards, the merged LSE stays [bs,hq,Lq]).
struct SeqLayoutIO { int rows_per_shard, heads, head0; };
// row0 > 0: only the rows [row0, Lq) of every batch are merged (and written); the tensors keep their full shapes.
int launch_lse_merge(const void* const* o_parts, const float* const* lse_parts, int n_parts, void* o_out,
                     float* lse_out, int bs, int64_t Lq, int hq, int hs, int part_dtype, int out_dtype,
                     hipStream_t stream, const SeqLayoutIO* seq = nullptr, int64_t row0 = 0);
// Optional: the running online-softmax state of a ring that delivers its blocks one call at a time (bf16 instance):
// attn_fwd_state_bytes() bytes in the kernel's own layout; first: the state is not read (the call starts it);
// last: the state is not written, the call writes the normalised O and the LSE instead.
struct RingState { float* state; int first, last; };
size_t attn_fwd_state_bytes(int bs, int64_t Lq, int hq, int hs);
int launch_ring_attn_fwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, void* o, float* lse, int bs, int64_t Lq,
                         int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc& qpos,
                         int in_dtype, int o_dtype, hipStream_t stream, const SeqLayoutIO* seq = nullptr,
                         const RingState* state = nullptr, bool v_transposed = false);
// The key-tile-transposed layout of V blocks (USP_SEQ_TO_HEAD_VT): bytes of one rank's block, and the launch that
// writes it for ranks rank_begin, rank_begin + rank_step, ... (packed back to back at dst when head_rank_base < 0,
// else indexed by rank - head_rank_base), straight from the sequence-layout shards.  bf16 data only.
inline size_t vt_block_bytes(int bs, int64_t Lk, int hkv, int hs) {
  return (size_t)bs * hkv * (size_t)((Lk + 63) / 64) * 64 * hs * 2;
}
int launch_layout_a2a_vt(const usp_problem& p, int heads, const void* src, void* dst, int rank_begin, int rank_end,
                         int head_rank_base, hipStream_t stream, int rank_step = 1);
// Key split: the same query rows against n_blocks blocks, every (query tile, head, batch, block) its own work item of
// ONE launch, each block's result (fp32 O, LSE) in its own partial, to be merged by launch_lse_merge.  Block j holds
// lk_blocks[j] <= Lk keys (all Lk when lk_blocks is null); Lk is the batch stride, in rows, of every block's tensors.
// With `mixed`, only the LAST n_split_tiles query tiles of the block (first in item order, the heaviest under a causal
// mask) are cut so; the other query tiles are whole items of the same launch that walk
// all blocks and write their finished rows (bf16, through `seq` when given) to mixed->o and mixed->lse.  The partials
// then hold the rows of the cut tiles only, to be merged over that row range.
// v_transposed: the V pointers are pieces of blocks in key-tile-transposed layout (each begins at a tile of 64 keys of
// its block; Lk, the batch stride in rows, then also gives the number of tiles per head of a whole block).
struct MixedLaunch { void* o; float* lse; int n_split_tiles; bool v_transposed; };
int launch_attn_fwd_partials(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                             const usp_posdesc* kpos_blocks, const int* lk_blocks, int n_blocks, float* const* o_parts,
                             float* const* lse_parts, int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int hs,
                             float scale, int causal, const usp_posdesc& qpos, hipStream_t stream,
                             const SeqLayoutIO* seq = nullptr, const MixedLaunch* mixed = nullptr);
int launch_block_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int bs, int64_t Lq,
                          int64_t Lk, int hq, int hkv, int hs, float scale, int causal, const usp_posdesc& qpos,
                          const usp_posdesc& kpos, int in_dtype, int o_dtype, hipStream_t stream);

// seq: o and d_o are the sequence-layout shards of the rank's Ulysses group (their first shard), not dense tensors.
int launch_bwd_delta(const void* o, const void* d_o, float* delta, int bs, int64_t L, int h, int hs,
                     hipStream_t stream, const SeqLayoutIO* seq = nullptr);
// How a backward launch pair divides its work (plan_bwd_cut): query heads of a KV group walked by one dK/dV
// workgroup, slices of a dQ item's key tiles, slices of a dK/dV item's query tiles.
struct BwdCut { int heads_per_wg, k_splits, q_splits; };
// equal_items: no causal mask (usp_attn_bwd knows; the per-call entry points, whose workspace query does not, say false).
BwdCut plan_bwd_cut(int bs, int64_t Lq, int64_t Lk, int hq, int hkv, int n_blocks, bool cut_items, bool equal_items);
// Room for copies of the outputs, one per slice: dq holds cut.k_splits copies dq_stride elements apart, every block's
// dk and dv hold (hq / hkv / cut.heads_per_wg) * cut.q_splits copies dkdv_stride elements apart; every copy is
// written (or added to, as the accumulate flags say) in full, nothing is atomic; launch_bwd_convert adds them up.
// ds (optional, null = off): room for the dS of one launch pair, bwd_ds_bytes() bytes: the dK/dV kernel then runs
// first and writes the dS blocks it forms, and the dQ kernel reads them back instead of forming S and dP again
// (5 matrix products per tile pair instead of 7, for 2 bytes written and read per visible pair).
struct BwdCopies { BwdCut cut; size_t dq_stride, dkdv_stride; void* ds = nullptr; };
inline bool bwd_keeps_ds(int hs) { return hs >= 128; }   // see plan_bwd
inline size_t bwd_ds_bytes(int bs, int64_t Lq, int64_t Lk, int hq, int n_blocks) {
  return (size_t)bs * hq * n_blocks * (size_t)((Lk + 255) / 256 * 8) * (size_t)((Lq + 255) / 256 * 8) * 2048;
}
int launch_ring_attn_bwd(const void* q, const void* const* k_blocks, const void* const* v_blocks,
                         const usp_posdesc* kpos_blocks, int n_blocks, const void* d_o, const float* lse,
                         const float* delta, float* dq, float* const* dk_blocks, float* const* dv_blocks, int bs,
                         int64_t Lq, int64_t Lk, int hq, int hkv, int hs, float scale, int causal,
                         const usp_posdesc& qpos, int accumulate_dq, const int* accumulate_dkdv, hipStream_t stream,
                         const struct BwdCopies* copies = nullptr);
int launch_block_attn_bwd(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                          const float* delta, float* dq, float* dk, float* dv, int bs, int64_t Lq, int64_t Lk, int hq,
                          int hkv, int hs, float scale, int causal, const usp_posdesc& qpos, const usp_posdesc& kpos,
                          int accumulate_dq, int accumulate_dkdv, hipStream_t stream);
// dst[i] = sum over n_copies of src[c * copy_stride + i], converted (fp32 output: optionally added to dst[i])
int launch_bwd_convert(const float* src, void* dst, size_t n, int out_dtype, hipStream_t stream, int n_copies = 1,
                       size_t copy_stride = 0, int add_to_dst = 0);
// The same for two tensors of the same size and copy layout in one launch (src1 == nullptr: one tensor).
int launch_bwd_convert2(const float* src0, void* dst0, const float* src1, void* dst1, size_t n, int out_dtype,
                        hipStream_t stream, int n_copies = 1, size_t copy_stride = 0, int add_to_dst = 0);
// The same with the result written to the sequence-layout shards of the rank's Ulysses group (seq; dst0 / dst1 = the
// group's first shard) instead of the dense [bs, rows, heads, hs] tensor the sources are: the reverse all-to-all of
// Algorithm 1 rides on the conversion's stores.  seq = null: dense, as above.
int launch_bwd_convert_seq(const float* src0, void* dst0, const float* src1, void* dst1, size_t n, int out_dtype,
                           hipStream_t stream, int n_copies, size_t copy_stride, int add_to_dst, const SeqLayoutIO* seq,
                           int bs, int64_t rows, int heads, int hs);

}  // namespace usp
