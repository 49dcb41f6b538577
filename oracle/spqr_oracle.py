"""Plain fp64 NumPy oracle of what the SpQR inference path computes.

TEST INFRASTRUCTURE: slow, obvious, independent of the HIP library.

The SpQR representation (Sec. 4.2) is a storage format, so the oracle is the
definition written out:

  1. per tile, read the four second-level 16-bit scalars s_s, z_s, s_z, z_z;
  2. per first-level group g, s_hat = dequantize(s_q, s_s, z_s) and
     z_hat = dequantize(z_q, s_z, z_z)            (Alg. 1, fit_statistics);
  3. per weight, W_hat = dequantize(Q, s_hat, z_hat) = s_hat * (Q - z_hat)
     (Alg. 1, dequantize), at every position, outlier positions included
     (the codes stay in place under outliers, Sec. 4.2);
  4. every CSR outlier (row, col, val) is added on top: W_hat[row, col] += val;
  5. y = W_hat @ x with x widened from fp16.

Reading of Alg. 1's fit_statistics, whose printed argument lists are
inconsistent: s_s, z_s are the scale / zero of the quantiser fitted to the
scales and s_z, z_z those of the quantiser fitted to the zeros, hence
s_hat = s_s * (s_q - z_s) and z_hat = s_z * (z_q - z_z).

Two variants of step 2 that the paper evaluates (Sec. 5, ablations), selected
by the optional attribute `stat_layout`:

  "round_zero"  the zero-point is a 3-bit integer: z_hat = z_q, used as it is;
                scales keep their second level (s_s, z_s), zeros have none;
  "stats16"     16-bit statistics: s_hat and z_hat are stored per group as
                16-bit floats (s16, z16); no codes, no second level.

Reading of "round zero": the text says the integer zero-point shrinks the
footprint, which it only does if the zeros' second-level pair (s_z, z_z) is
dropped, while the ablation table prints the unchanged 3.63 bits; the text is
followed.  (A matrix of the other reading is an ordinary bilevel one with
s_z = 1, z_z = 0, which decodes to the same values.)

Functions take the logical arrays produced by `spqr_synth` (attribute access
only: m, n, beta1, beta2, group_axis, Q, s_q, z_q, s_s, z_s, s_z, z_z,
row_ptr, col_idx, val, optional perm, stat_layout, s16, z16).
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# Alg. 1, dequantize:  s * (Q - z)
# --------------------------------------------------------------------------
def dequantize(q, s, z):
    return np.asarray(s, dtype=np.float64) * (np.asarray(q, dtype=np.float64)
                                             - np.asarray(z, dtype=np.float64))


def _tile_of_group(fmt):
    """How many group rows / group columns share one tile's second-level stats."""
    if fmt.group_axis == 0:       # groups [m, n/beta1]; a tile spans beta2 rows
        return fmt.beta2, 1
    return 1, fmt.beta2           # groups [m/beta1, n]; a tile spans beta2 columns


def _to_groups(t, fmt):
    """Broadcast a per-tile array to the per-group grid."""
    rr, cc = _tile_of_group(fmt)
    return np.repeat(np.repeat(t, rr, axis=0), cc, axis=1)


def stat_layout(fmt):
    return getattr(fmt, "stat_layout", "bilevel")


def decode_stats(fmt):
    """Step 2: first-level (s_hat, z_hat) per group, fp64 (Alg. 1 fit_statistics;
    Sec. 5 ablations for the two variants)."""
    lay = stat_layout(fmt)
    if lay == "stats16":
        return fmt.s16.astype(np.float64), fmt.z16.astype(np.float64)
    s_hat = dequantize(fmt.s_q, _to_groups(fmt.s_s, fmt), _to_groups(fmt.z_s, fmt))
    if lay == "round_zero":
        return s_hat, fmt.z_q.astype(np.float64)
    z_hat = dequantize(fmt.z_q, _to_groups(fmt.s_z, fmt), _to_groups(fmt.z_z, fmt))
    return s_hat, z_hat


def decode_stats_f32(fmt):
    """Decoded statistics in the precision a 32-bit device keeps them in.

    The paper does not fix the precision of the decoded statistics.  The
    reading taken here: code and second-level zero are widened to binary32,
    subtracted (one rounding), then multiplied by the second-level scale
    (one rounding); no fused multiply-add.
    """
    f = np.float32
    lay = stat_layout(fmt)
    if lay == "stats16":                    # a 16-bit float widens exactly
        return fmt.s16.astype(f), fmt.z16.astype(f)
    s_hat = (_to_groups(fmt.s_s, fmt).astype(f)
             * (fmt.s_q.astype(f) - _to_groups(fmt.z_s, fmt).astype(f))).astype(f)
    if lay == "round_zero":
        return s_hat, fmt.z_q.astype(f)
    z_hat = (_to_groups(fmt.s_z, fmt).astype(f)
             * (fmt.z_q.astype(f) - _to_groups(fmt.z_z, fmt).astype(f))).astype(f)
    return s_hat, z_hat


def _to_weights(g, fmt):
    """Broadcast a per-group array to the [m, n] weight grid."""
    if fmt.group_axis == 0:
        return np.repeat(g, fmt.beta1, axis=1)
    return np.repeat(g, fmt.beta1, axis=0)


def decode_dense(fmt):
    """Steps 1-3: the dense part, fp64 [m, n], no outliers."""
    s_hat, z_hat = decode_stats(fmt)
    return dequantize(fmt.Q, _to_weights(s_hat, fmt), _to_weights(z_hat, fmt))


def outlier_rows(fmt):
    """Row index of every CSR entry."""
    counts = np.diff(np.asarray(fmt.row_ptr, dtype=np.int64))
    return np.repeat(np.arange(fmt.m, dtype=np.int64), counts)


def add_outliers(W, fmt):
    """Step 4, in place: W[row, col] += val for every CSR entry."""
    if fmt.col_idx.shape[0]:
        np.add.at(W, (outlier_rows(fmt), fmt.col_idx.astype(np.int64)),
                  fmt.val.astype(np.float64))
    return W


def reconstruct(fmt):
    """Steps 1-4: W_hat including outliers, fp64 [m, n]."""
    return add_outliers(decode_dense(fmt), fmt)


def _permuted(X, fmt):
    """Activations in the stored column order: x'[j] = x[perm[j]].

    An act-order quantiser (Sec. 5 ablations; App. B `permutation_order
    act_order`) reorders the input dimension before Alg. 1's column sweep and
    stores the matrix in that order: stored column j is original column
    perm[j], hence W . x = sum_j W_stored[:, j] * x[perm[j]].
    """
    X = np.atleast_2d(np.asarray(X)).astype(np.float64)
    perm = getattr(fmt, "perm", None)
    if perm is not None:
        X = X[:, np.asarray(perm, dtype=np.int64)]
    return X


def matvec(fmt, X):
    """Step 5: Y[b, m] = X[b, :] . W_hat^T in fp64 (X is [b, n] or [n])."""
    return _permuted(X, fmt) @ reconstruct(fmt).T


def matvec_dense_only(fmt, X):
    return _permuted(X, fmt) @ decode_dense(fmt).T


def matvec_sparse_only(fmt, X):
    X = _permuted(X, fmt)
    Y = np.zeros((X.shape[0], fmt.m), dtype=np.float64)
    if fmt.col_idx.shape[0]:
        prod = X[:, fmt.col_idx.astype(np.int64)] * fmt.val.astype(np.float64)[None, :]
        rows = outlier_rows(fmt)
        for b in range(X.shape[0]):
            np.add.at(Y[b], rows, prod[b])
    return Y


def matvec_rows(fmt, X, rows):
    """Y[b, len(rows)] for selected output rows only (full-size spot checks)."""
    X = _permuted(X, fmt)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((X.shape[0], rows.shape[0]), dtype=np.float64)
    s_hat, z_hat = decode_stats(fmt)
    for k, i in enumerate(rows):
        if fmt.group_axis == 0:
            s_row = np.repeat(s_hat[i], fmt.beta1)
            z_row = np.repeat(z_hat[i], fmt.beta1)
        else:
            s_row = s_hat[i // fmt.beta1]
            z_row = z_hat[i // fmt.beta1]
        w = dequantize(fmt.Q[i], s_row, z_row)
        a, b = int(fmt.row_ptr[i]), int(fmt.row_ptr[i + 1])
        np.add.at(w, fmt.col_idx[a:b].astype(np.int64), fmt.val[a:b].astype(np.float64))
        out[:, k] = X @ w
    return out


# --------------------------------------------------------------------------
# App. D, Eq. 4: average bits per parameter of a configuration.
# --------------------------------------------------------------------------
def average_bits(b_w, b_s, b_z, beta1, beta2, r_o=0.0):
    return b_w + (b_s + b_z) / beta1 + 64.0 / (beta1 * beta2) + 32.0 * r_o


def average_bits_round_zero(b_w, b_s, b_z, beta1, beta2, r_o=0.0):
    """Eq. 4 with one second-level pair per tile instead of two (Sec. 5, "round zero")."""
    return b_w + (b_s + b_z) / beta1 + 32.0 / (beta1 * beta2) + 32.0 * r_o


def average_bits_stats16(b_w, beta1, r_o=0.0):
    """Eq. 4 for 16-bit first-level statistics and no second level (Sec. 5)."""
    return b_w + 32.0 / beta1 + 32.0 * r_o
