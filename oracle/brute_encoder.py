"""Alg. 1 (SpQRQuantize) once more, as scalar pure-Python loops over single weights, for tiny matrices.

TEST INFRASTRUCTURE.  Pins the vectorised oracle (spqr_encoder.py) against slips of indexing, masking and
broadcasting: Python floats are binary64, every step is one rounded operation, so the two must agree bit for
bit.  The readings are those listed in spqr_encoder.py.
"""
import math

import numpy as np


def _fit(vals, bits):
    """(s, z) of one group given as a list of floats (empty list: min = max = 0)."""
    lo = min(vals) if vals else 0.0
    hi = max(vals) if vals else 0.0
    s = (hi - lo) / float(2 ** bits - 1)
    if s == 0.0:
        s = 1.0
    return s, -lo / s, lo


def _quant(v, s, z, bits):
    return min(max(math.floor(v / s + z + 0.5), 0.0), float(2 ** bits - 1))


def _group_error(vals, hd, bits):
    """Total of the squared scaled rounding errors of one group, left to right."""
    s, z, _ = _fit(vals, bits)
    t = 0.0
    for v, h in zip(vals, hd):
        e = (v - s * (_quant(v, s, z, bits) - z)) / h
        t = t + e * e
    return t


def _second_level(stats, bits):
    """One group of beta2 first-level statistics -> (codes, s2, z2, de-quantised)."""
    s2, z2, lo = _fit(stats, bits)
    s2 = float(np.float16(s2))
    if s2 == 0.0:
        s2, z2 = 1.0, -lo
    z2 = float(np.float16(z2))
    codes = [_quant(v, s2, z2, bits) for v in stats]
    return codes, s2, z2, [s2 * (c - z2) for c in codes]


def spqr_quantize(W, Hic, bits, beta1, beta2, tau, s_bits=3, z_bits=3):
    W = [[float(v) for v in row] for row in np.asarray(W, dtype=np.float64)]
    U = np.asarray(Hic, dtype=np.float64)
    m, n = len(W), len(W[0])
    Q = [[0.0] * n for _ in range(m)]
    out = [[False] * n for _ in range(m)]
    ng = n // beta1
    Sq = [[0.0] * ng for _ in range(m)]; Zq = [[0.0] * ng for _ in range(m)]
    S2 = {k: [[0.0] * ng for _ in range(m // beta2)] for k in ("s_s", "z_s", "s_z", "z_z")}
    base_val = {}
    for g in range(ng):
        i = g * beta1
        hd = [float(U[j, j]) for j in range(i, i + beta1)]
        s1 = [0.0] * m; z1 = [0.0] * m
        for r in range(m):
            grp = W[r][i:i + beta1]
            base = _group_error(grp, hd, bits)
            for c in range(beta1):
                rest = grp[:c] + grp[c + 1:]
                ol = _group_error(rest, hd[:c] + hd[c + 1:], bits) if rest else 0.0
                out[r][i + c] = (base - ol) > tau
            kept = [grp[c] for c in range(beta1) if not out[r][i + c]]
            s1[r], z1[r], _ = _fit(kept, bits)
        s_hat = [0.0] * m; z_hat = [0.0] * m
        for t in range(m // beta2):
            rows = range(t * beta2, (t + 1) * beta2)
            cs, S2["s_s"][t][g], S2["z_s"][t][g], hs = _second_level([s1[r] for r in rows], s_bits)
            cz, S2["s_z"][t][g], S2["z_z"][t][g], hz = _second_level([z1[r] for r in rows], z_bits)
            for k, r in enumerate(rows):
                Sq[r][g], Zq[r][g], s_hat[r], z_hat[r] = cs[k], cz[k], hs[k], hz[k]
        for r in range(m):
            e = [0.0] * beta1
            for c in range(beta1):
                j = i + c
                Q[r][j] = _quant(W[r][j], s_hat[r], z_hat[r], bits)
                wq = s_hat[r] * (Q[r][j] - z_hat[r])
                e[c] = (W[r][j] - wq) / float(U[j, j]) * (0.0 if out[r][j] else 1.0)
                for k in range(j, i + beta1):
                    W[r][k] = W[r][k] - e[c] * float(U[j, k])
                if out[r][j]:
                    base_val[(r, j)] = wq
            for c in range(beta1):
                for k in range(i + beta1, n):
                    W[r][k] = W[r][k] - e[c] * float(U[i + c, k])
    entries = sorted(base_val)
    val = [np.float16(W[r][c] - base_val[(r, c)]) for r, c in entries]
    row_ptr = [0] * (m + 1)
    for r, _ in entries:
        row_ptr[r + 1] += 1
    for r in range(m):
        row_ptr[r + 1] += row_ptr[r]
    return dict(Q=np.array(Q), s_q=np.array(Sq), z_q=np.array(Zq), row_ptr=np.array(row_ptr),
                col_idx=np.array([c for _, c in entries], dtype=np.int64), val=np.array(val, dtype=np.float16),
                W_final=np.array(W), **{k: np.array(v) for k, v in S2.items()})
