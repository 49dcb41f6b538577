/*
 * Symbols libspqr.so exports for the library's own tests and tuning runs.  Not part of the public interface
 * (include/spqr.h): they may change or go away with any build.
 */
#ifndef SPQR_TEST_HOOKS_H_
#define SPQR_TEST_HOOKS_H_

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

#ifdef __cplusplus
}
#endif
#endif  /* SPQR_TEST_HOOKS_H_ */
