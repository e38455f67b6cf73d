/*
 * mlora_testing.h -- test and measurement switches of libmlora.
 *
 * Not part of the operator's interface (mlora.h): a process-wide switch that forces the slower
 * kernels, so that tests can compare every kernel mix on one shape, and a timing aid that
 * brackets the library's kernel launches with HIP events.  Unlike the entry points of mlora.h
 * the timing aid allocates: it creates HIP events (hipEventCreate) on first use and keeps them
 * until the process ends.  Production callers need neither.
 */
#ifndef MLORA_TESTING_H
#define MLORA_TESTING_H

#include "mlora.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Selects which kernels the entry points use (bit mask):
 *   0 (default) fastest applicable path: MFMA kernels when the problem is bf16, h and d are
 *               multiples of 64, every rank is a multiple of 8 and all buffers are 16-byte
 *               aligned; the generic kernels otherwise,
 *   bit 0       generic kernels for the two base products,
 *   bit 1       generic kernels for the low-rank products (3 = generic everywhere).
 * Returns the previous value.  Process-wide. */
int mlora_set_kernel_path(int path);

/* Measurement aid.  While enabled, every launch of the MFMA kernels by this process is bracketed
 * by a pair of HIP events recorded on the launch stream (at most 16384 launches are kept; the
 * events are created on first use and live until the process ends).  Returns the previous
 * setting. */
int mlora_profile_kernels(int enable);

/* Kinds of kernels the measurement aid tells apart, and the unit their work is counted in. */
#define MLORA_PROFILE_GEMM  0  /* base products with their LoRA steps; algorithmic flops
                                  (2 M N K plus 2 t_k r_k N per task)                          */
#define MLORA_PROFILE_ROWS  1  /* s x A and s dy B^T; algorithmic bytes (activation rows read
                                  once, result written once, adapter matrices read once)       */
#define MLORA_PROFILE_GRAD  2  /* dA_k and dB_k; algorithmic bytes                             */
#define MLORA_PROFILE_KINDS 3

/* Waits for the recorded launches to finish; for each kind returns the sum of their durations
 * in milliseconds, the sum of their work in that kind's unit, and their count, through the
 * non-NULL pointers (HOST arrays of MLORA_PROFILE_KINDS entries), and forgets them. */
mlora_status mlora_profile_kernels_read(double* ms_total, double* units_total, int* launches);

#ifdef __cplusplus
}
#endif
#endif /* MLORA_TESTING_H */
