// Calibration loops for the matrix-core roofline of the attention kernels: what the chip delivers on a loop
// that has the instruction mix of the forward kernel's steady state but none of its memory traffic, masks or
// bookkeeping.  Measurement aid only; nothing of the method (Algorithm 1) is computed here.
//
//   mode 0  pure MFMA: four independent v_mfma_f32_32x32x16_bf16 accumulation chains per wave, constant operands.
//   mode 1  attention mix: per wave and step 16 "score" MFMAs whose A operands are read from LDS as 16 B row
//           fragments, 16 "P V" MFMAs whose A operands come from LDS transpose reads and whose B operands are the
//           packed exp2 of the previous step's scores (32 fma + 32 exp2 + 16 pack + row sum per lane), operands read
//           two MFMAs ahead.  Pseudo-random operand bits: the matrix core's power draw, and with it the clock the
//           chip sustains, depends on the data.
// Both: 256 workgroups of 8 waves (two waves per SIMD), no global memory traffic inside the loop.
// Built into its own library (libusp_calib.so) that only bench.py loads: not part of the product's ABI.
#include "attn_device.h"
#include "calib_mfma.h"
#include "usp_internal.h"

namespace usp {
namespace {

using namespace dev;

constexpr int kCalibThreads = 512;
constexpr int kCalibGroups = 256;
constexpr int KT = 64, KSTR = 272, VSTR = 320;
constexpr int KBYTES = KT * KSTR, VBYTES = KT * VSTR;

__global__ __launch_bounds__(kCalibThreads) void calib_pure_mfma(float* sink, int iters) {
  bf16x8 x, y;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    x[e] = (__bf16)(0.001f * ((threadIdx.x + e) & 63));
    y[e] = (__bf16)(0.002f * ((threadIdx.x + 3 * e) & 63));
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  sink[blockIdx.x * kCalibThreads + threadIdx.x] = s;
}

__device__ inline bf16x8 calib_read_k(const char* krow, int i) {   // score MFMA i: k-step i / 2, key block i % 2
  return *(const bf16x8*)(krow + (i & 1) * 32 * KSTR + (i >> 1) * 32);
}
__device__ inline bf16x8 calib_read_v(const char* vlane, int j) {   // P V MFMA j: key step j / 4, dim block j % 4
  const char* p0 = vlane + (16 * (j >> 2)) * VSTR + (j & 3) * 64;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 8 * VSTR));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__global__ __launch_bounds__(kCalibThreads) void calib_attention_mix(float* sink, int iters) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  // bf16 pairs with random sign and mantissa, exponent of 0.5 .. 1
  for (int i = threadIdx.x; i < (2 * KBYTES + 2 * VBYTES) / 4; i += kCalibThreads) {
    uint32_t h = (i + blockIdx.x * 7919u) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    ((uint32_t*)lds)[i] = (h & 0x80ff80ffu) | 0x3f003f00u;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, l32 = lane & 31, hl = lane >> 5, grp = lane >> 4, j16 = lane & 15;
  bf16x8 q[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      q[j][e] = (__bf16)(0.37f * (float)((int)(((threadIdx.x * 2654435761u + e * 40503u + j * 9176u) >> 8) & 15) - 8));
  const int v_lane_off = (4 * hl + (j16 >> 2)) * VSTR + (16 * (grp & 1) + 4 * (j16 & 3)) * 2;
  f32x16 sa[2], sb[2], o[4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) { sa[j][i] = 0.01f * i; sb[j][i] = 0.f; }
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[j][i] = 0.f;
  float rowsum = 0.f;
  constexpr int D = 2;   // operands are read D MFMAs ahead
  auto step = [&](int it, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    const char* krow = lds + ((it + 1) & 1) * KBYTES + l32 * KSTR + hl * 16;
    const char* vlane = lds + 2 * KBYTES + (it & 1) * VBYTES + v_lane_off;
    bf16x8 frag[32 + D];
    u32x4 p[4];
#pragma unroll
    for (int i = 0; i < D; ++i) frag[i] = calib_read_k(krow, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i < 16) {
        const int ks = i >> 1, kbk = i & 1;
        f32x16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        sn[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i], q[ks], ks == 0 ? z : sn[kbk], 0, 0, 0);
      } else {
        const int j = i - 16;
        o[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i], __builtin_bit_cast(bf16x8, p[j >> 2]), o[j & 3], 0, 0, 0);
      }
      if (i + D < 32) frag[i + D] = (i + D) < 16 ? calib_read_k(krow, i + D) : calib_read_v(vlane, i + D - 16);
      if (i < 16) {
        const int b = i >> 3, e = (i & 7) * 2;
        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[b][e], 0.1f, -1.0f));
        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[b][e + 1], 0.1f, -1.0f));
        rowsum += e0 + e1;
        p[i >> 2][i & 3] = pack_bf16(e0, e1);
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the written order: MFMA, read-ahead, slice of the softmax
    }
  };
#pragma unroll 1
  for (int it = 0; it < iters; it += 2) {
    step(it, sa, sb);
    step(it + 1, sb, sa);
  }
  float s = rowsum;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += o[j][i];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += sa[j][i];
  sink[blockIdx.x * kCalibThreads + threadIdx.x] = s;
}

}  // namespace

static int launch_calib_mfma(int mode, int iters, float* sink, double* flop, hipStream_t stream) {
  iters &= ~1;   // the attention mix runs two steps per loop trip
  // every wave issues 32 MFMAs of 2 * 32 * 32 * 16 flop per iteration in both modes
  *flop = (double)kCalibGroups * (kCalibThreads / 64) * (double)iters * 32.0 * 32768.0;
  if (mode == 0) {
    hipLaunchKernelGGL(calib_pure_mfma, dim3(kCalibGroups), dim3(kCalibThreads), 0, stream, sink, iters);
    return launch_status();
  }
  constexpr size_t lds = 2 * KBYTES + 2 * VBYTES;
  static LdsLimitRaised lds_limit;   // per kernel instance
  if (!raise_dynamic_lds_limit((const void*)calib_attention_mix, lds, lds_limit)) return USP_ERR_LAUNCH;
  hipLaunchKernelGGL(calib_attention_mix, dim3(kCalibGroups), dim3(kCalibThreads), lds, stream, sink, iters);
  return launch_status();
}

}  // namespace usp

extern "C" __attribute__((visibility("default"))) int usp_calib_mfma(int mode, int iters, void* sink,
                                                                     size_t sink_bytes, double* flop, void* stream) {
  if (!sink || !flop) return USP_ERR_NULL;
  if (mode != 0 && mode != 1) return USP_ERR_UNSUPPORTED;
  if (iters < 2 || iters > (1 << 24)) return USP_ERR_SHAPE;
  if (sink_bytes < USP_CALIB_SINK_BYTES) return USP_ERR_WORKSPACE;
  return usp::launch_calib_mfma(mode, iters, (float*)sink, flop, (hipStream_t)stream);
}
