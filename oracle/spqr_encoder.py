"""Plain fp64 NumPy oracle of the SpQR quantiser (Alg. 1, SpQRQuantize and its subroutines).

TEST INFRASTRUCTURE: slow, obvious, independent of the HIP library.  Only tests, the smoke check and the
benchmark's CPU baseline call it.

Alg. 1 is an iteration with data-dependent integer decisions, so the oracle takes its steps in the paper's order
and notation.  Every floating-point step is one correctly rounded binary64 operation applied elementwise (no
library matrix product inside the sweep, sums written out left to right), which makes the integer outputs
(codes, statistic codes, the outlier set) reproducible bit for bit by any implementation that performs the same
operations in the same order.

Orientation: the paper's own (Alg. 1): a first-level group is beta1 consecutive columns of one row, the second
level groups the statistics of beta2 consecutive rows of one column block (`group_axis = 0`, tiles of
beta2 x beta1).

Readings (where the printed algorithm is silent, garbled or at odds with the text):

  Q1  H^ic is the UPPER triangular factor U of (H + lambda I)^-1 = U^T U: the sweep reads H^ic[j, j:], a row right of
      the diagonal.  lambda is added as printed (an absolute value, not a fraction of the mean diagonal).
  Q2  error(): `W_q := quantize(...)` followed by `W - W_q` only makes sense with W_q the de-quantised values;
      `/ H^ic` divides column j by the diagonal entry H^ic[j, j], as line 13 of the main loop does.
  Q3  outliers(): E_base has beta1 columns, E_ol beta1 - 1; "E_base - E_ol > tau" compares, per row, the group's total
      error with all weights quantised against its total error with weight i exempted (left out of the fit and
      of the error), which is the criterion of Sec. 4.1: a weight is an outlier if keeping it in 16 bit reduces
      the error by more than tau.  tau is absolute, as printed.
  Q4  fit_statistics(): "W * (1 - is_outlier)" is read with Sec. 4.1's sentence that the statistics are computed
      EXCLUDING outliers (App. B's fit_quantizer_without_outliers): outliers are left out of min / max, not
      replaced by zeros.  A group with nothing left has min = max = 0.
  Q5  fit_quantizer with max = min: s := 1, z := -min (code 0 de-quantises to min exactly).
  Q6  quantize clamps to [0, 2^bits - 1]: a code has `bits` bits, and columns are quantised with statistics that went
      through the second level and after the block's error feedback moved them, so values do leave the fitted
      range.
  Q7  The statistics' own quantisers use b_s and b_z bits (App. B), not the weights' b.
  Q8  The four second-level statistics are stored in 16 bits (Sec. 4.2): they are rounded to binary16 right after
      they are fitted, BEFORE the statistic codes are chosen and de-quantised, so that the decoder, which only
      sees the stored values, reconstructs exactly the s_hat, z_hat the sweep used.  A scale that rounds to 0 is
      treated like max = min (Q5).
  Q9  Line 16 prints H^ic[i:i+beta1, i:i+beta1]; the shapes require H^ic[i:i+beta1, i+beta1:n].  The product
      E . H^ic is evaluated as beta1 rank-one updates in column order j = i, i+1, ...
  Q10 gather_outlier_matrix: the format keeps a code under every outlier and adds the stored value on top of the
      de-quantised code (Sec. 4.2), so the stored value is binary16(W_final[r, c] - s_hat * (Q[r, c] - z_hat)),
      with W_final the weight as the sweep left it (adjusted by the error feedback of earlier columns).
  Q11 "act_order" (App. B's permutation_order; Sec. 5: "the GPTQ activation order heuristic") is named, not defined.
      Reading: the input columns are processed in the order of decreasing Hessian diagonal (the inputs with the
      largest second moments first), ties to the smaller index.  perm[j] is the original column that is processed
      and stored as column j: W and H are permuted before Alg. 1 runs and the stored matrix meets x[perm[j]] at
      inference (the decoder oracle's `perm`).
"""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np


def _f16(v):
    """Round binary64 to binary16 (nearest even) and widen back."""
    return np.asarray(v, dtype=np.float64).astype(np.float16).astype(np.float64)


# Alg. 1, line 2 / line 3 ---------------------------------------------------------------------------------------
def hessian(X):
    """H = 2 X X^T for calibration inputs X[n, d]."""
    X = np.asarray(X, dtype=np.float64)
    return 2.0 * (X @ X.T)


def inverse_cholesky(H, lam):
    """H^ic = Cholesky((H + lambda I)^-1), upper triangular: (H + lambda I)^-1 = H^ic^T H^ic  (Q1)."""
    H = np.asarray(H, dtype=np.float64)
    Hinv = np.linalg.inv(H + lam * np.eye(H.shape[0]))
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv).T.copy()


# Alg. 1, subroutines ---------------------------------------------------------------------------------------------
def fit_quantizer(M, bits, keep=None):
    """Min-max quantiser of every row of M (one group per row): s = (max - min) / (2^bits - 1), z = -min / s.
    keep: boolean mask of the entries that take part (Q4); Q5 for max = min."""
    M = np.asarray(M, dtype=np.float64)
    if keep is None:
        lo, hi = M.min(axis=1), M.max(axis=1)
    else:
        lo = np.where(keep, M, np.inf).min(axis=1)
        hi = np.where(keep, M, -np.inf).max(axis=1)
        none = ~keep.any(axis=1)
        lo = np.where(none, 0.0, lo)
        hi = np.where(none, 0.0, hi)
    s = (hi - lo) / float(2 ** bits - 1)
    flat = s == 0.0
    s = np.where(flat, 1.0, s)
    z = -lo / s
    return s, z


def quantize(M, s, z, bits):
    """floor(M / s + z + 0.5), clamped to the code range (Q6)."""
    q = np.floor(np.asarray(M, dtype=np.float64) / s + z + 0.5)
    return np.minimum(np.maximum(q, 0.0), float(2 ** bits - 1))


def dequantize(Q, s, z):
    return s * (Q - z)


def error(Wb, hdiag, bits):
    """Alg. 1 error(): squared, H^ic-scaled rounding error of a block whose rows are one group each (Q2)."""
    s, z = fit_quantizer(Wb, bits)
    Wq = dequantize(quantize(Wb, s[:, None], z[:, None], bits), s[:, None], z[:, None])
    E = (Wb - Wq) / hdiag[None, :]
    return E * E


def _row_sum(E):
    """Sum of the columns, left to right."""
    t = np.zeros(E.shape[0])
    for j in range(E.shape[1]):
        t = t + E[:, j]
    return t


def outliers(Wb, hdiag, bits, tau):
    """Alg. 1 outliers(): leave-one-out test of every weight of the block (Q3).  Returns the boolean mask."""
    m, b1 = Wb.shape
    base = _row_sum(error(Wb, hdiag, bits))
    mask = np.zeros((m, b1), dtype=bool)
    for i in range(b1):
        loo = [j for j in range(b1) if j != i]
        ol = _row_sum(error(Wb[:, loo], hdiag[loo], bits)) if loo else np.zeros(m)
        mask[:, i] = (base - ol) > tau
    return mask


def fit_second_level(v, beta2, bits):
    """Quantiser of a vector of first-level statistics in groups of beta2 consecutive rows, its two parameters
    rounded to binary16 (Q7, Q8).  Returns (codes, scale per group, zero per group, de-quantised statistics)."""
    g = v.reshape(-1, beta2)
    s2, z2 = fit_quantizer(g, bits)
    lo = g.min(axis=1)
    s2 = _f16(s2)
    flat = s2 == 0.0
    s2 = np.where(flat, 1.0, s2)
    z2 = _f16(np.where(flat, -lo, z2))
    codes = quantize(g, s2[:, None], z2[:, None], bits)
    hat = dequantize(codes, s2[:, None], z2[:, None])
    return codes.reshape(-1), s2, z2, hat.reshape(-1)


def fit_statistics(Wb, is_outlier, bits, beta2, s_bits, z_bits):
    """Alg. 1 fit_statistics() for one column block: first-level (s, z) per row without the outliers, then both
    vectors through the second level."""
    s, z = fit_quantizer(Wb, bits, keep=~is_outlier)
    s_q, s_s, z_s, s_hat = fit_second_level(s, beta2, s_bits)
    z_q, s_z, z_z, z_hat = fit_second_level(z, beta2, z_bits)
    return s_hat, z_hat, (s_q, z_q, s_s, z_s, s_z, z_z)


# Alg. 1, main procedure -----------------------------------------------------------------------------------------
def spqr_quantize(W, Hic, bits, beta1, beta2, tau, s_bits=3, z_bits=3):
    """SpQRQuantize from line 4 on (H^ic given).  W[m, n] binary64 (not modified), Hic[n, n] upper triangular.
    Returns the logical SpQR arrays (group_axis 0) and the weights as the sweep left them."""
    W = np.array(W, dtype=np.float64)
    Hic = np.asarray(Hic, dtype=np.float64)
    m, n = W.shape
    assert n % beta1 == 0 and m % beta2 == 0
    ng = n // beta1
    Q = np.zeros((m, n))
    E = np.zeros((m, n))
    O = np.zeros((m, n), dtype=bool)
    Sq = np.zeros((m, ng)); Zq = np.zeros((m, ng))
    Ss = np.zeros((m // beta2, ng)); Zs = np.zeros_like(Ss); Sz = np.zeros_like(Ss); Zz = np.zeros_like(Ss)
    Shat = np.zeros((m, ng)); Zhat = np.zeros((m, ng))
    for g, i in enumerate(range(0, n, beta1)):
        hdiag = np.diagonal(Hic)[i:i + beta1]
        O[:, i:i + beta1] = outliers(W[:, i:i + beta1], hdiag, bits, tau)                       # line 8
        s_hat, z_hat, st = fit_statistics(W[:, i:i + beta1], O[:, i:i + beta1], bits, beta2, s_bits, z_bits)  # line 9
        Sq[:, g], Zq[:, g], Ss[:, g], Zs[:, g], Sz[:, g], Zz[:, g] = st
        Shat[:, g], Zhat[:, g] = s_hat, z_hat
        for j in range(i, i + beta1):
            Q[:, j] = quantize(W[:, j], s_hat, z_hat, bits)                                     # line 11
            w_q = dequantize(Q[:, j], s_hat, z_hat)                                             # line 12
            E[:, j] = (W[:, j] - w_q) / Hic[j, j] * (1.0 - O[:, j])                             # line 13
            for k in range(j, i + beta1):                                                       # line 14
                W[:, k] = W[:, k] - E[:, j] * Hic[j, k]
        for j in range(i, i + beta1):                                                           # line 16 (Q9)
            if i + beta1 < n:
                W[:, i + beta1:] = W[:, i + beta1:] - E[:, j][:, None] * Hic[j, i + beta1:][None, :]
    # gather_outlier_matrix (Q10): CSR by row, then column
    rows, cols = np.nonzero(O)
    grp = cols // beta1
    base = dequantize(Q[rows, cols], Shat[rows, grp], Zhat[rows, grp])
    val = (W[rows, cols] - base).astype(np.float16)
    row_ptr = np.zeros(m + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=m), out=row_ptr[1:])
    return SimpleNamespace(
        m=m, n=n, w_bits=bits, s_bits=s_bits, z_bits=z_bits, beta1=beta1, beta2=beta2, group_axis=0,
        Q=Q.astype(np.uint8), s_q=Sq.astype(np.uint8), z_q=Zq.astype(np.uint8),
        s_s=Ss.astype(np.float16), z_s=Zs.astype(np.float16), s_z=Sz.astype(np.float16), z_z=Zz.astype(np.float16),
        row_ptr=row_ptr, col_idx=cols.astype(np.uint16), val=val, W_final=W, is_outlier=O, E=E, s_hat=Shat, z_hat=Zhat)


def act_order(H):
    """Q11: column order by decreasing diag(H), ties to the smaller index."""
    return np.argsort(-np.diagonal(np.asarray(H, dtype=np.float64)), kind="stable").astype(np.int32)


def spqr_quantize_act_order(W, X, bits, beta1, beta2, tau, lam, s_bits=3, z_bits=3):
    """SpQRQuantize with the activation-order heuristic: the result describes W[:, perm] and carries perm."""
    H = hessian(X)
    perm = act_order(H)
    r = spqr_quantize(np.asarray(W, dtype=np.float64)[:, perm], inverse_cholesky(H[np.ix_(perm, perm)], lam), bits, beta1,
                      beta2, tau, s_bits, z_bits)
    r.perm = perm
    return r


def spqr_quantize_from_calibration(W, X, bits, beta1, beta2, tau, lam, s_bits=3, z_bits=3):
    """SpQRQuantize(W, X, b, beta1, beta2, tau, lambda) as printed: lines 2-3, then the sweep."""
    return spqr_quantize(W, inverse_cholesky(hessian(X), lam), bits, beta1, beta2, tau, s_bits, z_bits)
