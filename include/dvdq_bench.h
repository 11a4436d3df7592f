/*
 * Measurement helpers exported by libdvdq next to the layer itself.  They are
 * not part of the quantized linear layer; the benchmark uses them to calibrate
 * its rooflines on the machine it runs on:
 *   - a plain copy kernel of known size (reference reading for the HBM traffic
 *     counters and for achievable copy bandwidth),
 *   - register-only MFMA loops, INT8 and FP6 (the matrix-core rate the chip sustains when
 *     nothing but MFMA issue limits it, and the rate it sustains on random 4-bit codes, where
 *     its power management lowers the clock).
 * Same conventions as dvdq.h: device pointers owned by the caller, work enqueued
 * on the caller's stream, DVDQ_OK or a dvdq_status code returned.
 */
#ifndef DVDQ_BENCH_H
#define DVDQ_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[i] = src[i] for `bytes` bytes (multiple of 16; both pointers 16-byte aligned). */
int dvdq_bench_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Every wave of a full-chip launch issues `iters` x 16 independent 32x32x32 INT8 MFMAs on
 * registers; `sink` (device, >= 4 bytes) receives a value that depends on the
 * result so the loop is not removed.  *ops_out (host pointer, may be NULL) receives the
 * number of integer operations (2 per multiply-add) the launch performs.
 * data: 0 = the same small constants in every lane and instruction; 1 = independent random codes in
 * [-7, 7] in every lane and operand register (4 x 4 operand pairs), which is the kind of data the layer
 * multiplies: how many operand bits change between instructions decides what the matrix cores draw and
 * with it the clock the chip holds.  Other values: DVDQ_ERR_UNSUPPORTED. */
int dvdq_bench_mfma_i8(int iters, int data, int32_t *sink, double *ops_out, void *hip_stream);

/* The same with `iters` x 8 independent 32x32x64 MFMAs on FP6 (E2M3) operands, the instruction the
 * W4A4 GEMM of the FP6 matrix path issues (data 1: 4 x 2 operand pairs of random codes as E2M3 patterns). */
int dvdq_bench_mfma_fp6(int iters, int data, int32_t *sink, double *ops_out, void *hip_stream);

/* Tile-configuration sweeps: force the native-layout GEMMs to use tile variant `variant`
 * (INT8 matrix path: 1..4, see the dispatch tables in w4ax_gemm.hip, one per code container; shapes too
 * shallow in K for a variant's ring fall back to variant 2.  FP6 matrix path: 1..2, see w4a4_fp6_gemm.hip,
 * other values mean its own choice); -1 restores the library's own choice.  Process-wide (an atomic
 * that every launch reads once), meant for benchmarking only. */
int dvdq_bench_set_gemm_variant(int variant);

/* How the native-layout GEMM's persistent workgroups get their tiles: 0 = fixed equal shares,
 * -1 = the library's own choice (tiles drawn from per-stream counters, fixed shares while a
 * stream is being captured).  Results are identical either way.  Process-wide (an atomic that every
 * launch reads once), meant for benchmarking only. */
int dvdq_bench_set_gemm_schedule(int schedule);

/* Experiments that share the chip between kernels: let the persistent GEMMs launch at most `workgroups`
 * workgroups (rounded down to a multiple of 8, at least 8) instead of filling every compute unit; 0 lifts the
 * limit.  Results are identical.  Process-wide (an atomic that every launch reads once), benchmarking only. */
int dvdq_bench_set_gemm_grid_limit(int workgroups);

/* Robustness tests: overwrite every word of the current GPU's tile counters with `value`, in stream
 * order on `hip_stream` (as a stray write or a launch that never finished would leave them).  GEMMs
 * launched afterwards must still give the right result. */
int dvdq_bench_fill_tile_counters(uint32_t value, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DVDQ_BENCH_H */
