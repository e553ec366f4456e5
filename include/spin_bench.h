/*
 * spin_bench.h -- measurement aids of the library declared in spin.h.  Nothing
 * here is part of the protocol: per-kernel HIP-event timing that benchmarks
 * switch on around a timed region, and a register-only int8 MFMA loop that
 * measures what the matrix cores sustain on given operand bytes.  Conventions
 * (device pointers, streams, return codes) as in spin.h.
 */
#ifndef SPIN_BENCH_H
#define SPIN_BENCH_H

#include "spin.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for benchmarks.  While enabled, every kernel the library
 * launches is bracketed by a pair of HIP events recorded on the caller's
 * stream; the events are created on demand, so while (and only while) timing
 * is enabled the library's calls do allocate event objects.  A launch on a
 * stream that is being captured into a HIP graph is not timed (recorded events
 * of a capture cannot be read), whatever the switch says.
 * spin_profile_read waits for the recorded events and returns the summed
 * duration in milliseconds and the number of launches of one kernel class
 * since the last spin_profile_reset.  The record is process-wide and guarded
 * by a mutex; spin_profile_reset must not run while another thread's timed
 * launches are still being enqueued. */
typedef enum {
    SPIN_KERNEL_RANDOM = 0,
    SPIN_KERNEL_SHARE = 1,
    SPIN_KERNEL_OPEN = 2,
    SPIN_KERNEL_BEAVER_MUL = 3,
    SPIN_KERNEL_TRUNC = 4,
    SPIN_KERNEL_PACK = 5,       /* open + digit split + fragment layout for the limb GEMM */
    SPIN_KERNEL_GEMM_LIMB = 6,
    SPIN_KERNEL_GEMM_VALU = 7,
    SPIN_KERNEL_LINCOMB = 8,
    SPIN_KERNEL_BINARY = 9,     /* bshare, bopen, beaver_and */
    SPIN_KERNEL_CAST = 10,      /* spin_cast_64_to_32 */
    SPIN_KERNEL_PROBE = 11,     /* spin_probe_mfma */
    SPIN_KERNEL_MUL_TRUNC = 12, /* spin_beaver_mul_trunc */
    SPIN_KERNEL_COUNT = 13
} spin_kernel;
void spin_profile_enable(int on);
spin_status spin_profile_read(int kernel, double *total_ms, unsigned *launches);
void spin_profile_reset(void);

/* Measurement aid: the int8 matrix-core rate the chip sustains on given operand bytes.  Every wave
 * of `blocks` workgroups (4 waves each) loads 24 MFMA operand fragments of 1 KiB from `operands`
 * ([24][128] uint64_t: 16 left fragments for two 32x32 tiles, then 8 right fragments; lane l of a wave
 * reads bytes 16 l .. 16 l + 15 of each) and issues, `iters` times, the 72 v_mfma_i32_32x32x32_i8 of one
 * k-step of the 64-bit limb GEMM (digit pairs i + j <= 7, pairs of one diagonal sharing an
 * accumulator), with no memory or LDS access inside the loop: blocks * 4 * iters * 72 * 65536 int8
 * operations per call.  sink[blocks * 256] receives each thread's wrapped int32 sum of its
 * accumulator registers, sign-extended (it keeps the loop alive and lets a test check the
 * arithmetic).  1 <= blocks <= 2^20, 1 <= iters <= 2^20.  Time it with spin_profile_* or events.  */
spin_status spin_probe_mfma(const uint64_t *operands, int blocks, int iters, uint64_t *sink,
                            spin_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SPIN_BENCH_H */
