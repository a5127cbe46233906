// N-way merge of the ring steps' partial results (blockwise attention of Sec. 2 combined over
// disjoint key blocks):  lse = ln sum_i exp(lse_i),  o = sum_i exp(lse_i - lse) * o_i.
//
// HBM-bound.  A workgroup owns kRows consecutive (position, head) rows of one batch entry.
// Phase 1: one thread per row reads the n partial LSEs (coalesced along the position axis of the
// [bs,hq,Lq] layout), computes the merged LSE and the n weights, and parks the weights in LDS.
// Phase 2: all threads stream the rows of every partial O as one contiguous range, 16 B per
// lane, accumulate in fp32 and write the merged O once.  Every byte is read once.
#include "usp_internal.h"

namespace usp {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 128;   // rows per workgroup

struct MergeArgs {
  const void* o[USP_MAX_MERGE_PARTS];
  const float* lse[USP_MAX_MERGE_PARTS];
  void* o_out;
  float* lse_out;
  int64_t Lq;
  int n_parts, hq, hs;
  int64_t rows_per_batch;   // Lq * hq
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

template <typename PartT, typename OutT>
__global__ __launch_bounds__(kThreads) void lse_merge_kernel(MergeArgs a) {
  extern __shared__ float w_lds[];   // [n_parts][kRows]
  const int b = blockIdx.y;
  const int64_t row0 = (int64_t)blockIdx.x * kRows;   // row = i * hq + h within the batch entry
  const int64_t rows_here = min((int64_t)kRows, a.rows_per_batch - row0);
  const int hq = a.hq, n = a.n_parts;

  // Phase 1.  Thread t handles the row with (h, i) such that consecutive threads walk i first.
  // The tile spans i in [i_lo, i_hi] and every h; rows outside [row0, row0+rows_here) are skipped.
  const int64_t i_lo = row0 / hq, i_hi = (row0 + rows_here - 1) / hq;
  const int ni = (int)(i_hi - i_lo + 1);
  for (int t = threadIdx.x; t < ni * hq; t += kThreads) {
    const int h = t / ni, di = t % ni;
    const int64_t i = i_lo + di;
    const int64_t row = i * hq + h;
    if (row < row0 || row >= row0 + rows_here) continue;
    const int64_t li = ((int64_t)b * hq + h) * a.Lq + i;
    float m = -INFINITY;
    for (int p = 0; p < n; ++p) m = fmaxf(m, a.lse[p][li]);
    const float ms = (m == -INFINITY) ? 0.0f : m;
    float tot = 0.0f;
    for (int p = 0; p < n; ++p) tot += __expf(a.lse[p][li] - ms);
    const float lse = tot > 0.0f ? ms + __logf(tot) : -INFINITY;
    const float inv = tot > 0.0f ? 1.0f / tot : 0.0f;
    const int lr = (int)(row - row0);
    for (int p = 0; p < n; ++p) w_lds[p * kRows + lr] = __expf(a.lse[p][li] - ms) * inv;
    a.lse_out[li] = lse;
  }
  __syncthreads();

  // Phase 2.  The tile's rows are contiguous in every [bs,Lq,hq,hs] tensor.
  const int vec_per_row = a.hs / 4;
  const int64_t tile_vecs = rows_here * vec_per_row;
  const int64_t elem0 = ((int64_t)b * a.rows_per_batch + row0) * a.hs;
  for (int64_t vi = threadIdx.x; vi < tile_vecs; vi += kThreads) {
    const int lr = (int)(vi / vec_per_row);
    const int64_t off = elem0 + vi * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int p = 0;
    // eight partial rows in flight per lane before the first multiply
    for (; p + 8 <= n; p += 8) {
      f32x4 x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = load4((const PartT*)a.o[p + j] + off);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float w = w_lds[(p + j) * kRows + lr];
        // a zero weight must erase the part even if it holds garbage (NaN payload of a skipped step)
        if (w != 0.f) acc += x[j] * w;
      }
    }
    for (; p < n; ++p) {
      f32x4 x = load4((const PartT*)a.o[p] + off);
      const float w = w_lds[p * kRows + lr];
      if (w != 0.f) acc += x * w;
    }
    store4((OutT*)a.o_out + off, acc);
  }
}

}  // namespace

int launch_lse_merge(const void* const* o_parts, const float* const* lse_parts, int n_parts, void* o_out,
                     float* lse_out, int bs, int64_t Lq, int hq, int hs, int part_dtype, int out_dtype,
                     hipStream_t stream) {
  MergeArgs a;
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
  a.rows_per_batch = Lq * hq;
  const int64_t gx = (a.rows_per_batch + kRows - 1) / kRows;
  if (gx > 0x7fffffffll || bs > 65535) return USP_ERR_UNSUPPORTED;
  dim3 grid((unsigned)gx, (unsigned)bs);
  const size_t lds = (size_t)n_parts * kRows * sizeof(float);
  if (part_dtype == USP_FP32 && out_dtype == USP_BF16)
    hipLaunchKernelGGL((lse_merge_kernel<float, __bf16>), grid, dim3(kThreads), lds, stream, a);
  else if (part_dtype == USP_FP32 && out_dtype == USP_FP32)
    hipLaunchKernelGGL((lse_merge_kernel<float, float>), grid, dim3(kThreads), lds, stream, a);
  else if (part_dtype == USP_BF16 && out_dtype == USP_BF16)
    hipLaunchKernelGGL((lse_merge_kernel<__bf16, __bf16>), grid, dim3(kThreads), lds, stream, a);
  else
    hipLaunchKernelGGL((lse_merge_kernel<__bf16, float>), grid, dim3(kThreads), lds, stream, a);
  return launch_status();
}

}  // namespace usp
