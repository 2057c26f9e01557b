/*
 * razer_tune.h -- launch-shape tuning hooks of the gfx950 RaZeR library.
 *
 * The paper's weight-only kernel is tuned offline: every matrix size is profiled ahead of time and the
 * number of SMs to launch is then picked per batch size when the kernel runs (Sec. 4.3; App. E, Tab. 13:
 * fewer, larger partitions cut the reduction stages of small problems).  The counterpart here: for a
 * problem (kernel family, activation rows m, weight rows, cols) the dispatch of razer_linear /
 * razer_linear_grouped takes its launch shape -- rows per workgroup, waves per K range, K-slices, which
 * of two kernels -- from a table compiled into the library (csrc/razer_tuned.inc), written by the
 * committed sweep `python -m paper_2501_04052_amd.tune` on the GPU; shapes that are not in the table
 * take a heuristic.  Results never depend on the shape beyond fp32 summation order.
 *
 * Families and their parameters p[0..3] (unused ones 0):
 *   RAZER_TUNE_GEMV         m = 1 (and 2 .. 4 with rows longer than 32768 elements): p[0] = groups of 2 rows
 *                           per set of waves (2, 4 or 8), p[1] = sets of waves per workgroup (1 or 2; 2 only
 *                           with p[0] = 2)
 *   RAZER_TUNE_GEMV_QUAD    m = 2 .. 4, every block size and weight format: p[0] = groups of 4 rows per
 *                           workgroup (4 or 8)
 *   RAZER_TUNE_SMALL_BATCH  5 <= m <= 32: p[0] = 0: K cut into slices over workgroups, summed by a second
 *                           launch from the workspace; p[1] = 128-element steps per slice (4 or 8), p[2] =
 *                           64-row blocks per workgroup (1, 2, 4).  p[0] = 1 (m <= 16 only): K inside the
 *                           workgroup, no workspace; p[1] = steps per wave and pass (1, 2), p[2] = groups of
 *                           16 rows per workgroup (1, 2, 3, 4, 8; 8 only with p[1] = 2)
 *   RAZER_TUNE_GEMM_SLICES  33 <= m <= 128: p[0] = K-slices of the register-decode kernel (1 .. 16)
 * For razer_linear_grouped `rows` is the sum over the group.  A shape the kernels are not built for is
 * ignored (the heuristic applies).
 */
#ifndef RAZER_TUNE_H
#define RAZER_TUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { RAZER_TUNE_GEMV = 0, RAZER_TUNE_GEMV_QUAD = 1, RAZER_TUNE_SMALL_BATCH = 2, RAZER_TUNE_GEMM_SLICES = 3,
       RAZER_TUNE_FAMILIES = 4 };

/* For the tuner: while set, every dispatch of `family` made by THIS host thread uses p[0..3] (HOST
 * array) instead of the table -- also razer_workspace_bytes, so size the workspace after forcing.
 * p = NULL clears the family's override; family = -1 with p = NULL clears all.  Returns 0, or 2 for a
 * bad family. */
int razer_tune_force(int family, const int32_t *p);

/* The shape the dispatch would use: copies it to p[0..3] (HOST) and returns 1 if it is this thread's
 * forced shape, 2 if it comes from the built-in table; returns 0 (p untouched) when the heuristic
 * applies. */
int razer_tune_lookup(int family, int64_t m, int64_t rows, int64_t cols, int32_t *p);

/* Number of entries of the built-in table. */
int razer_tune_table_size(void);

#ifdef __cplusplus
}
#endif
#endif /* RAZER_TUNE_H */
