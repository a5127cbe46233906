// Device-side helpers shared by the attention kernels (forward and backward): vector types for the MFMA
// operands, 32-bit position descriptors, bf16 packing and the half-wave combine.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace usp {
namespace dev {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Position descriptor narrowed to 32 bits (the host checks L < 2^31): fewer registers in the mask path.
struct PosDesc32 { int start0, len0, start1, len1; };
__device__ inline int pos_of(const PosDesc32& d, int i) { return i < d.len0 ? d.start0 + i : d.start1 + (i - d.len0); }
__device__ inline int pos_min(const PosDesc32& d, int a, int b) {
  int m = INT32_MAX;
  if (a < d.len0) m = d.start0 + a;
  if (b > d.len0) m = min(m, d.start1 + (max(a, d.len0) - d.len0));
  return m;
}
__device__ inline int pos_max(const PosDesc32& d, int a, int b) {
  int m = INT32_MIN;
  if (a < d.len0) m = d.start0 + min(b, d.len0) - 1;
  if (b > d.len0) m = max(m, d.start1 + (b - 1 - d.len0));
  return m;
}

// Tiles of a local index range that can hold a visible (query, key) pair: [a0,a1) then [b0,b1) (b may be empty).
struct TileRanges { int a0, a1, b0, b1; };

// Key tiles (of KT keys) visible to the query rows [row_lo, row_hi): under the causal rule kpos <= qpos the
// visible keys of each ascending run form a prefix of that run.
template <int KT>
__device__ inline TileRanges visible_key_tiles(int causal, const PosDesc32& qpos, const PosDesc32& kpos, int Lk,
                                               int row_lo, int row_hi) {
  TileRanges t;
  if (!causal) {
    t.a0 = 0; t.a1 = (Lk + KT - 1) / KT; t.b0 = t.b1 = t.a1;
    return t;
  }
  const int64_t qmax = pos_max(qpos, row_lo, row_hi);
  int64_t c0 = qmax - kpos.start0 + 1; c0 = c0 < 0 ? 0 : (c0 > kpos.len0 ? kpos.len0 : c0);
  int64_t c1 = qmax - kpos.start1 + 1; c1 = c1 < 0 ? 0 : (c1 > kpos.len1 ? kpos.len1 : c1);
  t.a0 = 0;
  t.a1 = (int)((c0 + KT - 1) / KT);
  if (c1 > 0) {
    t.b0 = (int)(kpos.len0 / KT);
    t.b1 = (int)(((int64_t)kpos.len0 + c1 + KT - 1) / KT);
    if (t.b0 < t.a1) t.b0 = t.a1;
    if (t.b1 < t.b0) t.b1 = t.b0;
  } else {
    t.b0 = t.b1 = t.a1;
  }
  return t;
}

// Query tiles (of QT rows) that see at least one key of [key_lo, key_hi): the rows of each ascending run
// with qpos >= the smallest key position form a suffix of that run.
template <int QT>
__device__ inline TileRanges visible_query_tiles(int causal, const PosDesc32& qpos, const PosDesc32& kpos, int Lq,
                                                 int key_lo, int key_hi) {
  TileRanges t;
  if (!causal) {
    t.a0 = 0; t.a1 = (Lq + QT - 1) / QT; t.b0 = t.b1 = t.a1;
    return t;
  }
  const int64_t kmin = pos_min(kpos, key_lo, key_hi);
  int64_t f0 = kmin - qpos.start0; f0 = f0 < 0 ? 0 : (f0 > qpos.len0 ? qpos.len0 : f0);   // first visible row of run 0
  int64_t f1 = kmin - qpos.start1; f1 = f1 < 0 ? 0 : (f1 > qpos.len1 ? qpos.len1 : f1);
  if (f0 < qpos.len0) {
    t.a0 = (int)(f0 / QT);
    t.a1 = (int)((qpos.len0 + QT - 1) / QT);
  } else {
    t.a0 = t.a1 = 0;
  }
  if (f1 < qpos.len1) {
    t.b0 = (int)((qpos.len0 + f1) / QT);
    t.b1 = (int)(((int64_t)qpos.len0 + qpos.len1 + QT - 1) / QT);
    if (t.b0 < t.a1) t.b0 = t.a1;
    if (t.b1 < t.b0) t.b1 = t.b0;
  } else {
    t.b0 = t.b1 = t.a1;
  }
  return t;
}

// Make a value that was loaded BEFORE a loop "arrive" here: the empty asm reads and redefines the register, so
// the compiler waits for the load at this point.  Without it the wait-count pass keeps the pre-loop load pending at
// the loop header and places its s_waitcnt vmcnt(n) at the first use INSIDE the loop, where, from the second trip
// on, it waits for that trip's freshly issued prefetch loads instead (the counter only knows "all but n").
__device__ inline void settle(bf16x8& x) {
  u32x4 t = __builtin_bit_cast(u32x4, x);
  asm volatile("" : "+v"(t));
  x = __builtin_bit_cast(bf16x8, t);
}
__device__ inline void settle(float& x) { asm volatile("" : "+v"(x)); }

__device__ inline uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Combine the two lane halves (lanes l and l ^ 32 hold the same query).  v_permlane32_swap(a, b) returns
// {a.lower | b.lower, a.upper | b.upper}; with a = b = x that is x of the lower half and x of the upper
// half, each broadcast to both halves.  (The two results are copied to scalars before the bit cast:
// a bit cast applied directly to a vector element reads element 0.)
__device__ inline float both_halves_max(float x) {
  const uint32_t xi = __builtin_bit_cast(uint32_t, x);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return fmaxf(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
__device__ inline float both_halves_sum(float x) {
  const uint32_t xi = __builtin_bit_cast(uint32_t, x);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return __builtin_bit_cast(float, lo) + __builtin_bit_cast(float, hi);
}

}  // namespace dev
}  // namespace usp
