/* Calibration of the matrix-core roofline: a measurement aid for bench.py, built into libusp_calib.so (not into the
 * product library, and not part of its ABI; it computes nothing of Algorithm 1).  Enqueues ONE launch of a loop that
 * touches no global memory until its last store:
 *   mode 0: independent v_mfma_f32_32x32x16_bf16 chains on constant operands;
 *   mode 1: the steady-state instruction mix of the forward block-attention kernel per wave and step
 *           (16 score MFMAs fed by 16 B LDS row reads, 16 P V MFMAs fed by LDS transpose reads, 32 exp2 and
 *           the bf16 packing of P) on pseudo-random operand bits (the clock the chip sustains depends on them).
 * 256 workgroups x 8 waves, `iters` steps each (rounded down to even, 2 <= iters <= 2^24).  `sink`: device
 * buffer of at least USP_CALIB_SINK_BYTES that receives one float per thread (sink_bytes is checked,
 * USP_ERR_WORKSPACE).  *flop (host) receives the MFMA flop of the launch: 2*32*32*16 per MFMA.  Status codes are
 * those of usp.h.  Timing is the caller's. */
#pragma once
#include <stddef.h>
#ifdef __cplusplus
extern "C" {
#endif
#define USP_CALIB_SINK_BYTES ((size_t)256 * 512 * 4)
int usp_calib_mfma(int mode, int iters, void* sink, size_t sink_bytes, double* flop, void* stream);
#ifdef __cplusplus
}
#endif
