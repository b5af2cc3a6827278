/*
 * skv_calib -- measurement aids for the benchmark of libskv; no part of the attention path.
 * Built as a library of its own (libskv_calib.so) so that the product library exports only the
 * path.  C linkage, device pointers, `stream` is a hipStream_t passed as void* (NULL = default).
 * Return value: 0 on success, 1 for an invalid argument, 7 if the launch failed.
 */
#ifndef SKV_CALIB_H
#define SKV_CALIB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Runs iters x 32 back-to-back v_mfma_f32_32x32x16_bf16 (32768 flop each) on every one of the
 * 4 * blocks waves of the launch (work groups of 256 threads, one wave per SIMD) and nothing else:
 * the rate the matrix cores of this device reach with the given operand values, the yardstick for
 * the pre-fill kernel's MFMA utilisation (the bf16 dense peak that the pre-fill phase of Sec. 3.1.1
 * is priced against).  operands: device, 16 KiB = 16 blocks of 64 lanes x 8 bf16 (A and B operand
 * of 8 steps; every instruction takes a different pair).  sink: device float[blocks * 256],
 * receives one value per lane so that the work cannot be dropped.  Asynchronous on `stream`; the
 * caller times it.  1 <= iters <= 2^20. */
int32_t skv_calib_mfma_bf16(const void *operands, float *sink, int32_t blocks, int32_t iters, void *stream);

/* The same MFMA stream with, between the MFMAs and independent of them, the other work a
 * flash-attention tile does per MFMA: mix bit 0 = four vector instructions per MFMA (three fma, one
 * exp2), bit 1 = LDS operand reads at the pre-fill kernel's rate (one 128-bit and two transposing
 * 64-bit reads per four MFMAs).  Nothing in it waits for anything, so a lower rate than
 * skv_calib_mfma_bf16's is the price of that work in power, i.e. in clock, and in issue slots.
 * The sink receives the same values as with mix = 0.  mix outside [0, 3] is an invalid argument. */
int32_t skv_calib_mfma_mix_bf16(const void *operands, float *sink, int32_t blocks, int32_t iters, int32_t mix,
                                void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SKV_CALIB_H */
