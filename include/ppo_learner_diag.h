/*
 * ppo_learner_diag.h - tracing and diagnostic aids of libppo_learner.so.
 *
 * Not part of the learner's path (include/ppo_learner.h declares that): a per-kernel-class
 * timer used by the benchmark's roofline report, and a direct call into the library's MFMA
 * GEMM tile kernel used by the tests.  Same conventions as ppo_learner.h.
 */
#ifndef PPO_LEARNER_DIAG_H
#define PPO_LEARNER_DIAG_H

#include "ppo_learner.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel-class timing (tracing aid, off by default).  ppo_profile(ctx, 1) clears the
 * counters and starts bracketing every kernel class launched by the calls above with HIP events
 * on the context's stream; ppo_profile(ctx, 0) stops.  ppo_profile_report synchronises and writes
 * one text line per class into the HOST buffer: "name launches total_ms algorithmic_flops
 * algorithmic_bytes"; returns the length written or a negative code. */
int ppo_profile(ppo_ctx* ctx, int32_t enable);
int64_t ppo_profile_report(ppo_ctx* ctx, char* h_buf, int64_t cap);

/* Diagnostic: C[M][N] (fp32, host) = A[M][K] * B[N][K]^T with A, B given as HOST fp32 and
 * narrowed to bf16, through the library's MFMA GEMM tile kernel.  K must be a multiple of 8. */
int ppo_diag_gemm(int32_t M, int32_t N, int32_t K, const float* h_a, const float* h_b, float* h_c);

/* Diagnostic: what a plain kernel reaches on the current GPU.  kind 0: streaming copy of nbytes with 16-byte
 * loads and stores (result: GB/s counting read + written bytes), 1: the read half alone, 2: the store half alone,
 * 3: the copy with non-temporal loads and stores, 4: a register-resident bf16 MFMA loop (result: TFLOP/s; nbytes
 * ignored), 5: a register-resident loop of one 16x16x32 bf16 MFMA followed by K = nbytes (0..8) independent vector
 * instructions, two waves per SIMD (result: TFLOP/s of the MFMAs; shows whether the two kinds of instruction overlap).
 * Allocates its own buffers, times `iters` launches with events on the default stream, synchronises. */
int ppo_diag_peak(int32_t kind, int64_t nbytes, int32_t iters, float* h_result);

#ifdef __cplusplus
}
#endif
#endif
