// N-way merge of the ring steps' partial results (blockwise attention of Sec. 2 combined over
// disjoint key blocks):  lse = ln sum_i exp(lse_i),  o = sum_i exp(lse_i - lse) * o_i.
//
// HBM-bound.  One thread per 16 B output vector: it first issues its loads of every partial O
// (nontemporal, up to 8 in flight), then works out the row's weights from the n partial LSEs while
// those loads fly, accumulates in fp32 and writes once.  The 32 (hs = 128) threads of a row repeat the
// weight arithmetic: a few dozen ALU instructions against 128+ B of traffic per thread, and no
// workgroup-level phase or barrier stands between the loads.  Measured on MI355X, one vector per
// thread streams ~15 % faster than a loop of several vectors per thread.
#include "usp_internal.h"

namespace usp {
namespace {

constexpr int kThreads = 256;

struct MergeArgs {
  const void* o[USP_MAX_MERGE_PARTS];
  const float* lse[USP_MAX_MERGE_PARTS];
  void* o_out;
  float* lse_out;
  int64_t Lq;
  int n_parts, hq, hs, bs;
  int64_t row0;             // first row that is merged (0 = all rows)
  int64_t rows_per_batch;   // (Lq - row0) * hq
  // SEQ instances: o_out is the first sequence-layout shard of the rank's Ulysses group, [U][bs][rows_per_shard]
  // [seq_heads][hs]; the rank's heads begin at seq_head0 (Algorithm 1's last all-to-all rides on the merge's stores)
  int rows_per_shard, seq_heads, seq_head0;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// streaming accesses: every byte is touched once, keep it out of the caches' way
__device__ inline f32x4 load4(const float* p) { return __builtin_nontemporal_load((const f32x4*)p); }
__device__ inline f32x4 load4(const __bf16* p) {
  bf16x4 v = __builtin_nontemporal_load((const bf16x4*)p);
  return __builtin_convertvector(v, f32x4);
}
__device__ inline void store4(float* p, f32x4 v) { __builtin_nontemporal_store(v, (f32x4*)p); }
__device__ inline void store4(__bf16* p, f32x4 v) {
  __builtin_nontemporal_store(__builtin_convertvector(v, bf16x4), (bf16x4*)p);
}

// NP = number of parts when it is at most 8 (everything unrolled, all loads in flight at once); NP = 0: any n.
template <typename PartT, typename OutT, int NP, bool SEQ>
__global__ __launch_bounds__(kThreads) void lse_merge_kernel(MergeArgs a) {
  const int vec_per_row = a.hs / 4;
  const int64_t vec = (int64_t)blockIdx.x * kThreads + threadIdx.x;      // over bs * rows_per_batch * vec_per_row
  const int64_t row_all = vec / vec_per_row;
  if (row_all >= a.rows_per_batch * a.bs) return;
  const int b = (int)(row_all / a.rows_per_batch);
  const int64_t row = row_all - (int64_t)b * a.rows_per_batch;           // row = i * hq + h
  const int64_t i = a.row0 + row / a.hq;
  const int h = (int)(row - (i - a.row0) * a.hq);
  const int64_t li = ((int64_t)b * a.hq + h) * a.Lq + i;
  const int64_t off = ((((int64_t)b * a.Lq + i) * a.hq + h) * vec_per_row + (vec - row_all * vec_per_row)) * 4;

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float lse_out;
  if constexpr (NP > 0) {
    // loads of O first, weights while they are in flight
    f32x4 x[NP];
    float l[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) x[p] = load4((const PartT*)a.o[p] + off);
#pragma unroll
    for (int p = 0; p < NP; ++p) l[p] = a.lse[p][li];
    float m = -INFINITY;
#pragma unroll
    for (int p = 0; p < NP; ++p) m = fmaxf(m, l[p]);
    const float ms = (m == -INFINITY) ? 0.0f : m;
    float tot = 0.0f;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      l[p] = __expf(l[p] - ms);      // exp(-inf) = 0 for dead parts
      tot += l[p];
    }
    const float inv = tot > 0.0f ? 1.0f / tot : 0.0f;
    lse_out = tot > 0.0f ? ms + __logf(tot) : -INFINITY;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const float w = l[p] * inv;
      // a zero weight must erase the part even if it holds garbage (NaN payload of a skipped step)
      const f32x4 t = x[p] * w;
      acc += (w != 0.f) ? t : f32x4{0.f, 0.f, 0.f, 0.f};
    }
  } else {
    const int n = a.n_parts;
    float m = -INFINITY;
    for (int p = 0; p < n; ++p) m = fmaxf(m, a.lse[p][li]);
    const float ms = (m == -INFINITY) ? 0.0f : m;
    float tot = 0.0f;
    for (int p = 0; p < n; ++p) tot += __expf(a.lse[p][li] - ms);
    const float inv = tot > 0.0f ? 1.0f / tot : 0.0f;
    lse_out = tot > 0.0f ? ms + __logf(tot) : -INFINITY;
    for (int p = 0; p < n; ++p) {
      const float w = __expf(a.lse[p][li] - ms) * inv;
      if (w != 0.f) acc += load4((const PartT*)a.o[p] + off) * w;
    }
  }
  int64_t out_off = off;
  if constexpr (SEQ) {
    const int64_t shard = i / a.rows_per_shard, s = i - shard * a.rows_per_shard;
    out_off = (((shard * a.bs + b) * a.rows_per_shard + s) * a.seq_heads + a.seq_head0 + h) * a.hs +
              (vec - row_all * vec_per_row) * 4;
  }
  store4((OutT*)a.o_out + out_off, acc);
  if (vec - row_all * vec_per_row == 0) a.lse_out[li] = lse_out;
}

template <typename PartT, typename OutT, bool SEQ = false>
void launch_typed(const MergeArgs& a, dim3 grid, hipStream_t stream) {
  switch (a.n_parts) {
#define USP_MERGE_CASE(N) \
  case N: hipLaunchKernelGGL((lse_merge_kernel<PartT, OutT, N, SEQ>), grid, dim3(kThreads), 0, stream, a); break;
    USP_MERGE_CASE(1) USP_MERGE_CASE(2) USP_MERGE_CASE(3) USP_MERGE_CASE(4)
    USP_MERGE_CASE(5) USP_MERGE_CASE(6) USP_MERGE_CASE(7) USP_MERGE_CASE(8)
#undef USP_MERGE_CASE
    default: hipLaunchKernelGGL((lse_merge_kernel<PartT, OutT, 0, SEQ>), grid, dim3(kThreads), 0, stream, a); break;
  }
}

}  // namespace

int launch_lse_merge(const void* const* o_parts, const float* const* lse_parts, int n_parts, void* o_out,
                     float* lse_out, int bs, int64_t Lq, int hq, int hs, int part_dtype, int out_dtype,
                     hipStream_t stream, const SeqLayoutIO* seq, int64_t row0) {
  if (row0 < 0 || row0 >= Lq) return USP_ERR_UNSUPPORTED;
  MergeArgs a;
  a.rows_per_shard = seq ? seq->rows_per_shard : 0;
  a.seq_heads = seq ? seq->heads : 0;
  a.seq_head0 = seq ? seq->head0 : 0;
  if (seq && part_dtype != USP_FP32) return USP_ERR_UNSUPPORTED;
  for (int i = 0; i < n_parts; ++i) {
    a.o[i] = o_parts[i];
    a.lse[i] = lse_parts[i];
  }
  a.o_out = o_out;
  a.lse_out = lse_out;
  a.Lq = Lq;
  a.n_parts = n_parts;
  a.hq = hq;
  a.hs = hs;
  a.row0 = row0;
  a.rows_per_batch = (Lq - row0) * hq;
  a.bs = bs;
  const int64_t vecs = (int64_t)bs * a.rows_per_batch * (hs / 4);
  const int64_t gx = (vecs + kThreads - 1) / kThreads;
  if (gx > 0x7fffffffll) return USP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)gx);
  if (seq && out_dtype == USP_BF16) launch_typed<float, __bf16, true>(a, grid, stream);
  else if (seq) launch_typed<float, float, true>(a, grid, stream);
  else if (part_dtype == USP_FP32 && out_dtype == USP_BF16) launch_typed<float, __bf16>(a, grid, stream);
  else if (part_dtype == USP_FP32 && out_dtype == USP_FP32) launch_typed<float, float>(a, grid, stream);
  else if (part_dtype == USP_BF16 && out_dtype == USP_BF16) launch_typed<__bf16, __bf16>(a, grid, stream);
  else launch_typed<__bf16, float>(a, grid, stream);
  return launch_status();
}

}  // namespace usp
