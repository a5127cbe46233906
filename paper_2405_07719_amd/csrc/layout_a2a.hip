// Ulysses all-to-all (Algorithm 1 steps 2-4 and 6) as a local permutation between the
// sequence layout [N][bs][L/N][heads][hs] and the head layout [N][bs][L/R][heads/U][hs].
//
// HBM-bound bit copy.  One (head-layout rank, batch, source shard u') slab is a set of L/N rows;
// on the head-layout side those rows are one contiguous range, on the sequence-layout side each
// row is a run of (heads/U)*hs elements at a stride of heads*hs.  Threads walk the slab in the
// head-layout (fully contiguous) order with the widest vector the run length allows, so both
// sides are accessed in whole runs: 1 KiB runs for 4 Q heads of size 128, 256 B for one KV head.
#include "usp_internal.h"

namespace usp {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 1;   // vectors per thread; measured on MI355X: 1 -> 6.1 TB/s, 4 -> 5.4 TB/s, 8 -> 3.9 TB/s

constexpr int kMaxTensors = USP_LAYOUT_MAX_TENSORS;

// Up to kMaxTensors tensors of one geometry (same heads, same ranks) go through one launch: on short sequences a
// launch costs as much as the copy itself (K and V of a rank; Q, O and dO of its backward; dK and dV).
struct LayoutArgs {
  const char* seq[kMaxTensors];    // sequence-layout buffer bases
  const char* head[kMaxTensors];   // head-layout buffer bases (slot of rank head_rank_base)
  int z_per_tensor;                // blockIdx.z values per tensor = ranks of the launch x batch
  int64_t n;           // rows per slab = L/N
  int64_t Lq;          // L/R
  int bs, U, rank_begin, rank_step, head_rank_base;
  // > 0: the launch covers whole Ulysses groups and the ranks of a group are dealt to NEIGHBOURING workgroups
  // (blockIdx.x = position * U + u): together they touch whole sequence-layout rows (all heads) at about the same
  // time, whole DRAM pages instead of one rank's 1 KiB run of every 8 KiB row per pass over the shard
  int interleave_u;
  uint32_t run_vecs;   // vectors per run = (heads/U)*hs*esize / sizeof(Vec)
  uint32_t row_vecs;   // vectors per sequence-layout row = heads*hs*esize / sizeof(Vec)
};

template <typename Vec, bool kToHead>
__global__ __launch_bounds__(kThreads) void layout_a2a_kernel(LayoutArgs a) {
  // blockIdx.z -> (tensor, rank, batch), blockIdx.y -> source shard u', blockIdx.x -> position in the slab
  const int tensor = (int)(blockIdx.z / a.z_per_tensor);
  const int z = (int)(blockIdx.z % a.z_per_tensor);
  const uint32_t bx = a.interleave_u ? blockIdx.x / (uint32_t)a.U : blockIdx.x;
  const int slot = a.interleave_u ? (z / a.bs) * a.U + (int)(blockIdx.x % (uint32_t)a.U) : z / a.bs;   // the slot-th rank of this launch
  const int rank = a.rank_begin + slot * a.rank_step;
  const int b = z % a.bs;
  const int up = (int)blockIdx.y;
  const int r = rank / a.U, u = rank % a.U;
  const uint64_t slab_vecs = (uint64_t)a.n * a.run_vecs;
  // head-layout side: whole buffers are indexed by rank; a packed workspace holds the launch's ranks back to back
  const uint64_t head_slot = a.head_rank_base < 0 ? (uint64_t)slot : (uint64_t)(rank - a.head_rank_base);
  const uint64_t head_row0 = head_slot * a.bs * a.Lq + (uint64_t)b * a.Lq + (uint64_t)up * a.n;
  Vec* head = (Vec*)a.head[tensor] + head_row0 * a.run_vecs;
  const uint64_t seq_row0 = ((uint64_t)(r * a.U + up) * a.bs + b) * a.n;
  Vec* seq = (Vec*)a.seq[tensor] + seq_row0 * a.row_vecs + (uint64_t)u * a.run_vecs;

  // One 32-bit division per thread; the following vectors step by kThreads with carried row / column.
  const uint32_t slab32 = (uint32_t)slab_vecs;
  const uint32_t base = bx * (uint32_t)(kThreads * kUnroll) + threadIdx.x;
  uint32_t row = base / a.run_vecs, col = base - row * a.run_vecs;
  const uint32_t drow = kThreads / a.run_vecs, dcol = kThreads - drow * a.run_vecs;
  uint64_t seq_off[kUnroll];
  Vec val[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    seq_off[i] = (uint64_t)row * a.row_vecs + col;
    row += drow;
    col += dcol;
    if (col >= a.run_vecs) {
      col -= a.run_vecs;
      ++row;
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const uint32_t idx = base + (uint32_t)i * kThreads;
    if (idx < slab32) val[i] = __builtin_nontemporal_load(kToHead ? seq + seq_off[i] : head + idx);
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const uint32_t idx = base + (uint32_t)i * kThreads;
    if (idx < slab32) __builtin_nontemporal_store(val[i], kToHead ? head + idx : seq + seq_off[i]);
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---- sequence layout -> key-tile-transposed head layout (V blocks for the attention kernel's P V product) --------
// Output per head-layout rank: [bs][heads/U][ceil(Lq/64) tiles][hs][64] bf16, where place j of a tile holds local row
// tile*64 + 16 (j / 16) + order(j % 16), order = 0-3, 8-11, 4-7, 12-15 (the order in which the two lane halves of the
// matrix instruction's 16-key step hold their keys); rows past Lq are zeros.  Still a pure permutation of Algorithm
// 1's all-to-all, with the transposition the attention kernel would otherwise do at every read of a tile.
// One thread moves an 8 x 8 block: 8 rows (the 8 keys of one 16-byte output chunk) x 8 head dims: eight 16-byte
// loads, a transposition of 16-bit elements in registers (v_perm_b32), eight 16-byte stores.
struct LayoutVtArgs {
  const uint16_t* seq;
  uint16_t* vt;
  int64_t n, Lq;       // rows per shard, rows per ring block
  int bs, U, heads, hl, hs;   // all heads of the sequence layout, heads per rank
  int rank_begin, rank_step, head_rank_base;
  int n_tiles;         // ceil(Lq / 64)
  int64_t total;       // threads with work: slots * bs * hl * n_tiles * hs
};

__global__ __launch_bounds__(kThreads) void layout_a2a_vt_kernel(LayoutVtArgs a) {
  const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (t >= a.total) return;
  const int per_tile = a.hs;                     // (hs / 8 dim chunks) x 8 output chunks
  const int in_tile = (int)(t % per_tile);
  int64_t w = t / per_tile;
  const int tile = (int)(w % a.n_tiles); w /= a.n_tiles;
  const int h = (int)(w % a.hl); w /= a.hl;
  const int b = (int)(w % a.bs);
  const int slot = (int)(w / a.bs);
  const int dchunk = in_tile % (a.hs / 8), jc = in_tile / (a.hs / 8);   // 8 head dims; output chunk = places 8 jc .. + 7
  const int rank = a.rank_begin + slot * a.rank_step;
  const int r = rank / a.U, u = rank % a.U;
  // the 8 local rows of output chunk jc: group of 16 = jc / 2, half = jc % 2 -> rows 4 half .. + 3 and 8 + 4 half .. + 3
  const int row_base = tile * 64 + 16 * (jc >> 1) + 4 * (jc & 1);
  u32x4 in[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int64_t i = row_base + (k & 3) + 8 * (k >> 2);
    if (i < a.Lq) {
      const int64_t up = i / a.n, srow = i - up * a.n;
      const uint16_t* src = a.seq + ((((int64_t)(r * a.U + up) * a.bs + b) * a.n + srow) * a.heads + (u * a.hl + h)) * a.hs + dchunk * 8;
      in[k] = __builtin_nontemporal_load((const u32x4*)src);
    } else {
      in[k] = u32x4{0, 0, 0, 0};
    }
  }
  const int64_t head_slot = a.head_rank_base < 0 ? slot : rank - a.head_rank_base;
  uint16_t* dst = a.vt + ((((head_slot * a.bs + b) * a.hl + h) * a.n_tiles + tile) * a.hs + dchunk * 8) * 64 + jc * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // output row = head dim dchunk * 8 + e: element e of each of the 8 input rows
    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;   // high or low halves of (second, first)
    u32x4 out;
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) out[wd] = __builtin_amdgcn_perm(in[2 * wd + 1][e >> 1], in[2 * wd][e >> 1], sel);
    __builtin_nontemporal_store(out, (u32x4*)(dst + e * 64));
  }
}

template <typename Vec>
int launch_vec(LayoutArgs a, int dir, size_t run_bytes, size_t row_bytes, int n_ranks, int n_tensors, hipStream_t stream) {
  a.run_vecs = (uint32_t)(run_bytes / sizeof(Vec));
  a.row_vecs = (uint32_t)(row_bytes / sizeof(Vec));
  const uint64_t slab_vecs = (uint64_t)a.n * a.run_vecs;
  const uint64_t gx = (slab_vecs + (uint64_t)kThreads * kUnroll - 1) / ((uint64_t)kThreads * kUnroll);
  // the kernel indexes a slab with 32 bits (a slab is one rank's share of one shard: far below 4 Gi vectors)
  if (slab_vecs + (uint64_t)kThreads * kUnroll >= (1ull << 32) || (uint64_t)n_tensors * n_ranks * a.bs > 65535ull ||
      a.U > 65535)
    return USP_ERR_UNSUPPORTED;
  a.z_per_tensor = n_ranks * a.bs;
  dim3 grid((unsigned)gx, (unsigned)a.U, (unsigned)(n_tensors * n_ranks * a.bs));
  a.interleave_u = 0;
  // Measured on MI355X, all ranks of a workload's Q (1 KiB runs, U 8): head -> seq 5.65 -> 6.32 TB/s at L = 212992 and
  // 5.87 -> 6.15 at L = 32768; seq -> head gains at the first (6.03 -> 6.35) and loses at the second (6.03 -> 5.58),
  // U = 2 (4 KiB runs) loses 6-8 % both ways, 256 B runs are even: so only the scattering direction, U >= 4, runs of
  // 512 B and more.
  if (dir == USP_HEAD_TO_SEQ && a.U >= 4 && run_bytes >= 512 && a.rank_step == 1 && a.rank_begin % a.U == 0 &&
      n_ranks % a.U == 0 && gx * (uint64_t)a.U < (1ull << 31)) {
    a.interleave_u = 1;
    a.z_per_tensor = (n_ranks / a.U) * a.bs;
    grid = dim3((unsigned)(gx * a.U), (unsigned)a.U, (unsigned)(n_tensors * (n_ranks / a.U) * a.bs));
  }
  if (dir == USP_SEQ_TO_HEAD)
    hipLaunchKernelGGL((layout_a2a_kernel<Vec, true>), grid, dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((layout_a2a_kernel<Vec, false>), grid, dim3(kThreads), 0, stream, a);
  return launch_status();
}

}  // namespace

int launch_layout_a2a_vt(const usp_problem& p, int heads, const void* src, void* dst, int rank_begin, int rank_end,
                         int head_rank_base, hipStream_t stream, int rank_step) {
  if (p.dtype != USP_BF16 || p.hs % 8) return USP_ERR_UNSUPPORTED;
  if (((uintptr_t)src | (uintptr_t)dst) & 15) return USP_ERR_UNSUPPORTED;
  const int N = p.ulysses * p.ring;
  LayoutVtArgs a;
  a.seq = (const uint16_t*)src;
  a.vt = (uint16_t*)dst;
  a.n = p.L / N;
  a.Lq = p.L / p.ring;
  a.bs = p.bs; a.U = p.ulysses; a.heads = heads; a.hl = heads / p.ulysses; a.hs = p.hs;
  a.rank_begin = rank_begin; a.rank_step = rank_step; a.head_rank_base = head_rank_base;
  a.n_tiles = (int)((a.Lq + 63) / 64);
  const int n_ranks = (rank_end - rank_begin + rank_step - 1) / rank_step;
  a.total = (int64_t)n_ranks * a.bs * a.hl * a.n_tiles * a.hs;
  const int64_t gx = (a.total + kThreads - 1) / kThreads;
  if (gx > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(layout_a2a_vt_kernel, dim3((unsigned)gx), dim3(kThreads), 0, stream, a);
  return launch_status();
}

int launch_layout_a2a(const usp_problem& p, int heads, int dir, const void* src, void* dst, int rank_begin,
                      int rank_end, int head_rank_base, hipStream_t stream, int rank_step) {
  return launch_layout_a2a_multi(p, heads, dir, 1, &src, &dst, rank_begin, rank_end, head_rank_base, stream, rank_step);
}

int launch_layout_a2a_multi(const usp_problem& p, int heads, int dir, int n_tensors, const void* const* src,
                            void* const* dst, int rank_begin, int rank_end, int head_rank_base, hipStream_t stream,
                            int rank_step) {
  if (n_tensors < 1 || n_tensors > kMaxTensors) return USP_ERR_UNSUPPORTED;
  const size_t es = dtype_size(p.dtype);
  const int N = p.ulysses * p.ring;
  LayoutArgs a;
  uintptr_t align = 0;
  for (int t = 0; t < kMaxTensors; ++t) {
    const int tt = t < n_tensors ? t : 0;
    a.seq[t] = (const char*)(dir == USP_SEQ_TO_HEAD ? src[tt] : dst[tt]);
    a.head[t] = (const char*)(dir == USP_SEQ_TO_HEAD ? dst[tt] : src[tt]);
    align |= (uintptr_t)src[tt] | (uintptr_t)dst[tt];
  }
  a.n = p.L / N;
  a.Lq = p.L / p.ring;
  a.bs = p.bs;
  a.U = p.ulysses;
  a.rank_begin = rank_begin;
  a.rank_step = rank_step;
  a.head_rank_base = head_rank_base;
  const size_t run_bytes = (size_t)(heads / p.ulysses) * p.hs * es;
  const size_t row_bytes = (size_t)heads * p.hs * es;
  align |= run_bytes;
  const int n_ranks = (rank_end - rank_begin + rank_step - 1) / rank_step;
  if (align % 16 == 0) return launch_vec<u32x4>(a, dir, run_bytes, row_bytes, n_ranks, n_tensors, stream);
  if (align % 8 == 0) return launch_vec<u32x2>(a, dir, run_bytes, row_bytes, n_ranks, n_tensors, stream);
  if (align % 4 == 0) return launch_vec<uint32_t>(a, dir, run_bytes, row_bytes, n_ranks, n_tensors, stream);
  return launch_vec<uint16_t>(a, dir, run_bytes, row_bytes, n_ranks, n_tensors, stream);
}

}  // namespace usp
