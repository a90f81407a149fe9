/*
 * atomo_bench.h - measurement helpers of libatomo (not part of the method): HIP-event timing of the library's
 * kernel launches by class, work counters of the Jacobi SVD, and the achievable fp32 matrix-core rate of the
 * GPU.  Benchmarks use them; an application that only encodes and decodes needs atomo.h alone.
 */
#ifndef ATOMO_BENCH_H
#define ATOMO_BENCH_H

#include "atomo.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Work counters as read by the most recent atomo_status call (host-side only): how many 64x64
 * block-pair eigenproblems the Jacobi SVD solved since the status call before it, how many
 * Jacobi steps (32 disjoint plane rotations each) those took in total, and how many 64-row x
 * 64-column tiles of the data the row updates of the data-space matrices rotated (pairs that
 * were found converged are left alone and not counted). */
int atomo_last_counters(const atomo_ctx* ctx, int32_t* pair_visits /*host*/, int32_t* jacobi_steps /*host*/,
                        int32_t* row_update_tiles /*host*/);

/* Kernel classes whose GPU time can be measured with HIP events (for benchmarks; not part of the
 * method).  While profiling is on, every launch of these kernels is bracketed by two events on the
 * caller's stream, which costs a few microseconds per launch. */
enum {
    ATOMO_K_SVD_PREPARE = 0, ATOMO_K_SVD_GRAM, ATOMO_K_SVD_EIG, ATOMO_K_SVD_UPDATE, ATOMO_K_SVD_REFRESH,
    ATOMO_K_SVD_FINALIZE,
    ATOMO_K_DECODE_SVD, ATOMO_K_EW_HIST, ATOMO_K_EW_SOLVE, ATOMO_K_EW_SAMPLE, ATOMO_K_EW_DECODE,
    ATOMO_K_SVD_THIN,
    ATOMO_K_COUNT
};

/* Switches event bracketing on (enable != 0) or off and discards what was collected. */
int atomo_profile_enable(atomo_ctx* ctx, int enable);

/* Waits for the recorded events, then adds to total_ms[k] / launches[k] (HOST arrays of
 * ATOMO_K_COUNT entries, caller-initialised) the GPU time and the number of bracketed launches of
 * each kernel class since the last read. */
int atomo_profile_read(atomo_ctx* ctx, double* total_ms, int64_t* launches);

/* What a loop of nothing but fp32 matrix-core instructions (v_mfma_f32_32x32x2f32, four independent accumulators
 * per wave, 16 waves per compute unit) reaches on this GPU, in TFLOP/s: the achievable figure to set beside the
 * published peak.  Runs two short kernels on `stream` and waits for them (about a millisecond). */
int atomo_measure_mfma_fp32(atomo_ctx* ctx, double* tflops /*host*/, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ATOMO_BENCH_H */
