/*
 * spqr_encode.h - C ABI of the SpQR quantiser (Alg. 1, SpQRQuantize) for AMD MI355X (gfx950).
 *
 * Produces the logical arrays of the Sparse-Quantized Representation (Sec. 4.2) from a weight matrix W[m, n]
 * and calibration inputs X[n, d], in the paper's own orientation (spqr.h: group_axis 0 - a first-level group is
 * beta1 consecutive columns of one row, the second level joins the statistics of beta2 consecutive rows of one
 * column block).  spqr_pack_host (spqr.h) turns the arrays into the packed layout the product kernels read.
 *
 * The three steps of Alg. 1, one entry point each:
 *   spqr_hessian           line 2:   H = 2 X X^T
 *   spqr_inverse_cholesky  line 3:   H^ic = Cholesky((H + lambda I)^-1), the UPPER factor: (H + lambda I)^-1 =
 *                                    H^ic^T H^ic (the sweep reads row j of H^ic from the diagonal to the right)
 *   spqr_quantize          lines 4-20: per column block the leave-one-out outlier test (outliers()), the bilevel
 *                                    statistic fit without the outliers (fit_statistics()), and the column sweep:
 *                                    quantize, E = (W - w_q) / H^ic_jj (0 at outliers), W -= E . H^ic
 *   spqr_gather_outliers   line 19:  the outlier set as CSR arrays, by row, then by column
 *   spqr_act_order, spqr_permute_columns, spqr_permute_symmetric: the activation-order heuristic around it (App. B)
 *
 * Arithmetic: binary64 throughout.  spqr_quantize performs exactly one correctly rounded binary64 operation per
 * step of the algorithm, elementwise, sums and updates in column order, never fused: given the same W, H^ic and
 * parameters its integer outputs (codes, statistic codes, outlier set) and the stored 16-bit values are a pure
 * function of the inputs, reproducible bit for bit.  spqr_hessian and spqr_inverse_cholesky are ordinary
 * floating-point linear algebra (blocked, fused multiply-adds): accurate to rounding, not order-exact.
 *
 * Conventions where Alg. 1 is silent or garbled:
 *   - quantize(v, s, z) = min(max(floor(v / s + z + 0.5), 0), 2^bits - 1);
 *   - fit_quantizer with max = min gives s = 1, z = -min; a group with no weight left after the outliers are
 *     taken out has min = max = 0;
 *   - the statistics' own quantisers use s_bits / z_bits; their two parameters are rounded to binary16 (the
 *     stored precision) BEFORE the statistic codes are chosen and de-quantised, so the decoder reconstructs the
 *     s_hat, z_hat the sweep used; a second-level scale that rounds to 0 becomes s = 1, z = binary16(-min);
 *   - the outlier test compares, per row, the group's summed error with all beta1 weights quantised against the
 *     summed error with weight i left out of both the fit and the sum: outlier iff the difference > tau
 *     (tau absolute); errors are (w - dequantize(quantize(w))) / H^ic_jj, squared;
 *   - an outlier keeps its code; its stored value is binary16(w_final - s_hat * (Q - z_hat)), w_final being the
 *     weight as the error feedback of earlier columns left it (Sec. 4.2: outlier values are added on top of the
 *     de-quantised code).
 *
 * Pointers are DEVICE pointers.  All calls are asynchronous on the given HIP stream (hipStream_t as void*, NULL =
 * default stream), allocate nothing, free nothing and never synchronise: scratch comes from the caller.  Returns
 * SPQR_OK or a negative spqr_status (spqr.h).
 */
#ifndef SPQR_ENCODE_H_
#define SPQR_ENCODE_H_

#include <stddef.h>
#include <stdint.h>

#include "spqr.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Alg. 1 line 2.  X[n][d] row-major (row j = the d calibration values of input j), H[n][n] row-major, both
 * binary64, 8-byte aligned; H is overwritten (both triangles).  n, d >= 1 (SPQR_ERR_SHAPE otherwise). */
int spqr_hessian(const double* X, int32_t n, int32_t d, double* H, void* stream);

/* Scratch of spqr_inverse_cholesky in bytes (two square matrices of n rounded up to 64, and the inverses of the
 * diagonal blocks); 0 if n < 1. */
size_t spqr_inverse_cholesky_workspace_bytes(int32_t n);

/* Alg. 1 line 3.  H[n][n] row-major, symmetric (the lower triangle is read), Hic[n][n] row-major: the upper
 * triangular factor with positive diagonal, zeros below it.  H and Hic may not overlap.  workspace: 256-byte
 * aligned, at least spqr_inverse_cholesky_workspace_bytes(n) bytes (SPQR_ERR_WORKSPACE if smaller).  H + lambda I
 * must be positive definite: otherwise Hic holds NaNs (nothing is reported: no synchronisation). */
int spqr_inverse_cholesky(const double* H, int32_t n, double lambda, double* Hic, void* workspace,
                          size_t workspace_bytes, void* stream);

/* The activation-order heuristic (App. B: `permutation_order act_order`; Sec. 5 ablations), which the paper names
 * without defining it; reading taken: the input columns are quantised in the order of decreasing Hessian diagonal
 * (the inputs with the largest second moments first), ties to the smaller index.  perm[j] (n entries, int32) = the
 * original column that is processed and STORED as column j: the caller quantises spqr_permute_columns(W, perm) with
 * the factor of spqr_permute_symmetric(H, perm) and hands `perm` to the product calls (spqr_matrix_t::perm), which
 * multiply stored column j with x[perm[j]].  workspace: 256-byte aligned, spqr_act_order_workspace_bytes(n) bytes.
 * n <= 65536.  The order is a pure function of diag(H): bit-exact against a stable sort. */
size_t spqr_act_order_workspace_bytes(int32_t n);
int spqr_act_order(const double* H, int32_t n, int32_t* perm, void* workspace, size_t workspace_bytes, void* stream);
/* W_out[i][j] = W[i][perm[j]] (m x n, row-major binary64; W_out != W). */
int spqr_permute_columns(const double* W, int32_t m, int32_t n, const int32_t* perm, double* W_out, void* stream);
/* H_out[i][j] = H[perm[i]][perm[j]] (n x n; H_out != H). */
int spqr_permute_symmetric(const double* H, int32_t n, const int32_t* perm, double* H_out, void* stream);

/* What spqr_quantize writes (all caller-allocated, sizes in elements):
 *   Q            uint8  [m][n]               codes in [0, 2^w_bits)
 *   s_q, z_q     uint8  [m][n/beta1]         statistic codes in [0, 2^s_bits), [0, 2^z_bits)
 *   s_s,z_s,s_z,z_z  binary16 bits [m/beta2][n/beta1]   second-level statistics, one per tile
 *   outlier_mask uint8  [m][n]               1 where the weight is an outlier
 *   outlier_val  binary16 bits [m][n]        the stored value at outlier positions, 0 elsewhere
 *   row_ptr      int32  [m+1]                exclusive prefix of the outlier counts per row; row_ptr[m] = nnz
 *   W_final      binary64 [m][n] or NULL     the weights as the sweep left them (quantised values at ordinary
 *                                            positions, adjusted full-precision weights at outliers)
 * Q, outlier_mask 4-byte aligned, outlier_val 4-byte aligned, n a multiple of 4. */
typedef struct spqr_quantized_t {
  uint8_t* Q;
  uint8_t* s_q;
  uint8_t* z_q;
  uint16_t* s_s;
  uint16_t* z_s;
  uint16_t* s_z;
  uint16_t* z_z;
  uint8_t* outlier_mask;
  uint16_t* outlier_val;
  int32_t* row_ptr;
  double* W_final;
} spqr_quantized_t;

/* Scratch of spqr_quantize in bytes: a column-major binary64 working copy of W. */
size_t spqr_quantize_workspace_bytes(int32_t m, int32_t n);

/* Alg. 1 lines 4-20 (H^ic given).  W[m][n] row-major binary64 (read only), Hic[n][n] from
 * spqr_inverse_cholesky.  w_bits in [2, 8], s_bits, z_bits in [1, 8]; beta1 in {4, 8, 16, 32}; beta2 a power of two in
 * [2, 64]; m a multiple of beta2, n a multiple of beta1 (SPQR_ERR_PARAM / SPQR_ERR_SHAPE otherwise).  workspace:
 * 256-byte aligned, spqr_quantize_workspace_bytes(m, n) bytes.  tau = +infinity switches the outlier test off. */
int spqr_quantize(const double* W, const double* Hic, int32_t m, int32_t n, int32_t w_bits, int32_t s_bits,
                  int32_t z_bits, int32_t beta1, int32_t beta2, double tau, const spqr_quantized_t* out,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Alg. 1 line 19: the CSR arrays of the outlier set from spqr_quantize's mask, values and row_ptr.  col_idx and
 * val hold row_ptr[m] entries (the caller reads that count after synchronising, then allocates); n <= 65536. */
int spqr_gather_outliers(const uint8_t* outlier_mask, const uint16_t* outlier_val, const int32_t* row_ptr,
                         int32_t m, int32_t n, uint16_t* col_idx, uint16_t* val, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPQR_ENCODE_H_ */
