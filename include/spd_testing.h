/*
 * Test hooks of the spd library.  They take HOST pointers and touch no GPU, so the host
 * logic (the planner, and the per-visit products and expansion functions shared with the
 * kernels) can be checked on a machine without one.  spd_pairwise / spd_knn never call
 * them and never compute on the CPU.
 */
#ifndef SPD_TESTING_H
#define SPD_TESTING_H

#include <stddef.h>
#include <stdint.h>

#include "spd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One distance from two sparse rows (host arrays, ascending columns), evaluated the way
 * the kernels do: row norms, the product g(a, b) over the stored entries of `b` with `a`
 * looked up by column (0 when absent), then the expansion function (Table 1; Section 2.2,
 * Eq. 2 in its single-sweep form).  Returns SPD_ERR_* on bad arguments. */
spd_status spd_host_pair_value(spd_metric metric, float p, int64_t n_cols, const int32_t *a_cols,
                               const float *a_vals, int64_t a_len, const int32_t *b_cols,
                               const float *b_vals, int64_t b_len, float *out);

/* Runs the planner on two row-pointer arrays (host) exactly as spd_pairwise / spd_knn
 * would (`k_neighbors` = 0 for pairwise), checks the plan's consistency, and writes a
 * JSON summary (staging kind, rows per group, workgroup size, LDS bytes, spilled rows,
 * slabs, chunks) into `json` (at most `cap` bytes, always terminated).
 * `options`: n_options pairs name/value as for spd_set_option. */
spd_status spd_host_plan_summary(const int64_t *a_indptr, int64_t a_rows, const int64_t *b_indptr,
                                 int64_t b_rows, int64_t n_cols, spd_metric metric, int k_neighbors,
                                 const char *const *option_names, const int64_t *option_values,
                                 int n_options, char *json, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* SPD_TESTING_H */
