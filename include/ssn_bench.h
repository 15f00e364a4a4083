/*
 * ssn_bench.h -- measurement aids of libssn_hip.so.  Not part of the method's interface (that is ssn.h):
 * bench.py uses them to time single kernels with HIP events on the library's own stream.
 */
#ifndef SSN_BENCH_H
#define SSN_BENCH_H

#include "ssn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid for benchmarks: launches ONE kernel of the hot path `reps` times back to back on the
 * context's stream between two HIP events and returns the mean duration of a launch in milliseconds.
 *   which = 0  the kernel of ssn_objective (margins + loss over all rows)
 *           1  first kernel of ssn_gradient: two-kernel path margins + U = P - Y; one-pass path margins,
 *              U and the per-workgroup partials of X^T U in a single sweep over X
 *           2  second kernel of ssn_gradient: two-kernel path X^T U per-chunk partials; one-pass path the
 *              fixed-order sum of the partials (+ lambda W)
 *           3, 4  the same two kernels of ssn_hess_apply on the prepared sample
 *           5  a plain streaming read of the whole data matrix (no arithmetic): the practical HBM ceiling
 * M [dev] is the p-by-K right operand (W or V).  which = 2 / 4 reuse what which = 1 / 3 left behind, so
 * call those first.  ms [host].  Synchronises the stream. */
int ssn_time_kernel(ssn_ctx *ctx, int32_t which, const void *M, int32_t reps, double *ms);

/* Which kernels serve this context: 0 = CSR, 1 = dense two-kernel path (margins, then X^T U), 2 = dense
 * one-pass path (every row of X read once per product; needs K <= 16 and p <= 1024; rows need no alignment
 * beyond their element's), 3 = dense binary path (C = 2, at least 128 features: matrix-vector kernels on the
 * vector units, margins then X^T u).
 * The environment variable SSN_DENSE_PATH=split forces 1 at ssn_create, SSN_BINARY_PATH=mfma keeps a binary
 * problem on the matrix-core paths, and SSN_SAMPLED_SLICES=0 turns off the feature-sliced margins of sampled
 * products on wide matrices (all three for measurements). */
int ssn_dense_path(const ssn_ctx *ctx);

/* Feature slices of the last sampled product's margins kernel on the two-kernel dense path (dense_zpart_kernel, with
 * dense_xtu_kernel forming U from the slices' partial margins); 0: the plain kernels served it. */
int ssn_sampled_slices(const ssn_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SSN_BENCH_H */
