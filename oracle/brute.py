"""Brute-force pure-Python decode of a logical SpQR matrix (tiny inputs only).

TEST INFRASTRUCTURE.  One weight at a time, with explicit index arithmetic, so
that the vectorised oracle's broadcasting can be checked against it.
Follows Sec. 4.2 (representation) and Alg. 1 (dequantize, fit_statistics).
"""


def weight(fmt, i, j):
    """Dense-part value of W_hat[i, j] (no outliers), Python floats (binary64)."""
    b1, b2 = fmt.beta1, fmt.beta2
    if fmt.group_axis == 0:
        gi, gj = i, j // b1          # group: row i, column block j // beta1
        ti, tj = i // b2, j // b1    # tile: beta2 rows of that column block
    else:
        gi, gj = i // b1, j          # group: row block i // beta1, column j
        ti, tj = i // b1, j // b2    # tile: beta2 columns of that row block
    lay = getattr(fmt, "stat_layout", "bilevel")
    if lay == "stats16":             # Sec. 5: statistics kept in 16 bit per group
        s_hat, z_hat = float(fmt.s16[gi, gj]), float(fmt.z16[gi, gj])
    else:
        s_hat = float(fmt.s_s[ti, tj]) * (int(fmt.s_q[gi, gj]) - float(fmt.z_s[ti, tj]))
        if lay == "round_zero":      # Sec. 5: the zero-point is the integer code
            z_hat = float(int(fmt.z_q[gi, gj]))
        else:
            z_hat = float(fmt.s_z[ti, tj]) * (int(fmt.z_q[gi, gj]) - float(fmt.z_z[ti, tj]))
    return s_hat * (int(fmt.Q[i, j]) - z_hat)


def reconstruct(fmt):
    W = [[weight(fmt, i, j) for j in range(fmt.n)] for i in range(fmt.m)]
    for i in range(fmt.m):
        for k in range(int(fmt.row_ptr[i]), int(fmt.row_ptr[i + 1])):
            W[i][int(fmt.col_idx[k])] += float(fmt.val[k])
    return W


def matvec(fmt, x):
    """y[i] = sum_j W_hat[i, j] * x[j] for a single vector x (length n)."""
    W = reconstruct(fmt)
    xs = [float(v) for v in x]
    if getattr(fmt, "perm", None) is not None:
        xs = [xs[int(p)] for p in fmt.perm]
    return [sum(W[i][j] * xs[j] for j in range(fmt.n)) for i in range(fmt.m)]
