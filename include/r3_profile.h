/*
 * r3_profile.h - measurement aids of the replayed-routing MoE library.
 *
 * Not part of the method (include/r3.h is): per-kernel timing of the library's
 * own launches with HIP events, and three calibration kernels that bench.py
 * uses to put the rooflines into context.  Unlike the method's calls these
 * keep process-wide state: pools of HIP events, created on first use and kept,
 * and an on/off flag; r3_profile_enable and r3_profile_read take a lock.  With
 * profiling off a kernel launch reads the flag and touches nothing else.
 */
#ifndef R3_PROFILE_H
#define R3_PROFILE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid (not part of the method): per-kernel timing with HIP events
 * recorded on the launch stream.  r3_profile_enable(1) clears the counters and
 * starts recording (at most 512 launches per kernel are kept), (0) stops.
 * r3_profile_read waits for the recorded events and returns the summed
 * duration in milliseconds and the number of launches of kernel `tag`
 * (0 <= tag < r3_profile_tags()); r3_profile_name names it.
 */
int r3_profile_enable(int on);
int r3_profile_tags(void);
const char *r3_profile_name(int tag);
int r3_profile_read(int tag, double *total_ms, int *launches);

/*
 * Measurement aid: a plain device-to-device copy kernel (`calib_copy_kernel`)
 * of `bytes` bytes (a multiple of 16; dst and src 16-byte aligned device
 * pointers, not overlapping).  It reads `bytes` and writes `bytes` of HBM and
 * nothing else, so hardware traffic counters read for it give the factor that
 * converts those counters to bytes for the other kernels of the same run.
 */
int r3_profile_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Measurement aid: a pure bf16 MFMA issue loop (`calib_mfma_kernel`, one
 * work-group of 8 waves per compute unit, 8 independent 32x32x16 accumulator
 * tiles per wave, operands in registers, no memory traffic) of `iters`
 * iterations; random_operands != 0 fills the operand registers with varied bit
 * patterns, 0 with one constant.  It does 2*32*32*16 * 8 * iters * 8 * grid
 * FLOP (r3_profile_mfma_flops); timed by the caller it gives the matrix rate
 * this machine sustains under its power limit, which depends on the operand
 * data.  `sink` is a device float the kernel may write (never in practice).
 */
int r3_profile_mfma(int iters, int random_operands, float *sink, void *stream);
double r3_profile_mfma_flops(int iters);

/*
 * Measurement aid: the same MFMA loop fed the way the expert GEMMs feed theirs
 * (`calib_mix_kernel`): per 8 MFMAs a wave reads 6 fragments from LDS, and per
 * 16 MFMAs of each wave the work-group brings 32 KB into LDS with direct
 * global->LDS loads from `src_1mib` (device, 1 MiB, 16-byte aligned, finite
 * bf16 values; stays cache-resident).  No barriers, epilogues or HBM misses:
 * the rate a perfect schedule of that instruction mix reaches under the power
 * limit.  Same FLOP count as r3_profile_mfma (r3_profile_mfma_flops).
 * shape 0: the kernels' shape, 8 waves of 128 x 64 per work-group.  shape 1: 4
 * waves of 128 x 128 (8 fragment reads per 16 MFMAs, the same global->LDS
 * bytes per FLOP): the ceiling of the other shape the GEMM header can be built
 * for.  Any other shape: R3_ERR_INVALID_ARG.
 */
int r3_profile_gemm_mix(int shape, int iters, const void *src_1mib, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* R3_PROFILE_H */
