/*
 * Symbols libspqr.so exports for the library's own tests and tuning runs.  Not part of the public interface
 * (include/spqr.h): they may change or go away with any build.
 */
#ifndef SPQR_TEST_HOOKS_H_
#define SPQR_TEST_HOOKS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Launch plan of the matrix-core path of spqr_gemm_smallbatch / spqr_gemm_fused; host arithmetic only, no
 * device is touched.  The dense launch walks every strip of tiles in steps of 64 tiles; `groups` workgroups
 * (4 or 8 strips each) cover the rows, and the `nsteps` steps of a group are split among workgroups of `s`
 * steps each (the last one may get fewer), every split writing a partial result.  Returns the s the library
 * takes, 1 <= s <= nsteps: the one whose simulated schedule is shortest, where the workgroups start in grid
 * order (split by split: the groups, behind those of the first split the `long_workgroups` workgroups of the
 * long outlier rows) on the first free of `slots` places on the chip (`slots_one_step` places when s == 1:
 * that kernel variant is smaller); a dense workgroup costs its steps + 0.3, a long-row workgroup 0.45 (0.02
 * behind later splits, where it leaves at once), every split 0.3 for its partial result; ties go to fewer
 * splits.  Candidates are s <= 32 and s = nsteps; a candidate whose launch has more than 200000 workgroups is
 * passed over.  The option SPQR_OPT_BATCH_STEPS pins s = min(value, nsteps).
 * A negative return is an SPQR_ERR_* code (an argument below 1, or long_workgroups below 0). */
int spqr_plan_batch_steps(int groups, int nsteps, int slots_one_step, int slots, int long_workgroups);

/* Plan of ONE launch of spqr_gemv_grouped for `count` (1..8) matrices of one format (w_bits, beta1, beta2,
 * group_axis, layout_version; 3-bit statistic codes, or 16-bit statistics for layout 3), matrix i being m[i] x n[i]
 * with nnz[i] outliers and the hint max_row_nnz[i]; host arithmetic only, no device is touched.  The matrices of
 * the width n[0] size the launch (the library sorts the width with the most strips to the front before it plans).
 * `max_waves` and `slots` describe the kernel instance: the wavefronts a workgroup may have and the wavefronts a
 * compute unit holds (from the kernel's register count at run time); `row_dots_on_matrix_cores` says whether the
 * instance keeps its row dot products on the matrix cores (3-bit, 8 x 32 tiles, group_axis 1).
 * Returns the number of table entries k (the matrices taken; the others wait for the next launch), in grid order:
 * entries[7 * j + 0..6] = matrix index, strips per workgroup R, wavefronts per strip P, outlier chunks per round,
 * 1 if the outlier products take the place of x, the chunks the LDS behind x holds then, workgroups of the entry.
 * *wavefronts = R * P of every entry, *lds_bytes = the launch's dynamic LDS.  Negative: an SPQR_ERR_* code
 * (SPQR_ERR_PARAM also where no plan exists). */
int spqr_plan_grouped(int count, const int32_t* m, const int32_t* n, const int32_t* max_row_nnz, const int64_t* nnz,
                      int w_bits, int beta1, int beta2, int group_axis, int layout_version, int max_waves, int slots,
                      int row_dots_on_matrix_cores, int32_t* entries, int32_t* wavefronts, int64_t* lds_bytes);

#ifdef __cplusplus
}
#endif
#endif  /* SPQR_TEST_HOOKS_H_ */
