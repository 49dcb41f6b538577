"""Pins for the CPU oracle: closed forms, printed values, invariants, special
cases that reduce to library routines, and brute force on tiny inputs.

None of these re-type the oracle's own formula; each would fail for a plausible
mistake (dropped zero-point, wrong sign, swapped second-level statistics,
transposed grouping, mis-indexed tile, outliers replacing instead of adding).
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import spqr_synth as synth
from oracle import brute, encoder_primitives as enc, spqr_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(m=32, n=32, **kw):
    kw.setdefault("seed", (7, m, n))
    return synth.make_matrix(m, n, **kw)


# ---- P1: hand-computed values, exactly representable --------------------------
def test_single_tile_hand_values():
    # One 16x16 tile.  s_s=0.5, z_s=1, s_q=3 -> s_hat = 0.5*(3-1) = 1.0
    # s_z=0.25, z_z=2, z_q=4 -> z_hat = 0.25*(4-2) = 0.5 ; q=5 -> w = 1.0*(5-0.5) = 4.5
    for axis in (0, 1):
        f = tiny(16, 16, group_axis=axis, outlier_rate=0.0)
        f.Q[:] = 5
        f.s_q[:] = 3
        f.z_q[:] = 4
        f.s_s[:] = 0.5; f.z_s[:] = 1.0; f.s_z[:] = 0.25; f.z_z[:] = 2.0
        W = orc.reconstruct(f)
        assert np.all(W == 4.5)
        # distinguish the four second-level scalars: change one at a time
        f.z_s[:] = 2.0              # s_hat = 0.5*(3-2) = 0.5 ; w = 0.5*(5-0.5) = 2.25
        assert np.all(orc.reconstruct(f) == 2.25)
        f.z_z[:] = 0.0              # z_hat = 0.25*4 = 1.0 ; w = 0.5*(5-1) = 2.0
        assert np.all(orc.reconstruct(f) == 2.0)
        f.s_z[:] = 1.0              # z_hat = 4 ; w = 0.5*(5-4) = 0.5
        assert np.all(orc.reconstruct(f) == 0.5)
        f.s_s[:] = -2.0             # s_hat = -2*(3-2) = -2 ; w = -2*(5-4) = -2
        assert np.all(orc.reconstruct(f) == -2.0)


def test_group_and_tile_indexing_hand_values():
    # 32x32 with beta1=8, beta2=16: mark ONE group / ONE tile and check which
    # weights move.  axis 0: group = row i, columns [8c, 8c+8); tile = 16 rows x 8 cols.
    f = tiny(32, 32, beta1=8, beta2=16, group_axis=0, outlier_rate=0.0)
    f.Q[:] = 1; f.s_q[:] = 1; f.z_q[:] = 0
    f.s_s[:] = 1.0; f.z_s[:] = 0.0; f.s_z[:] = 1.0; f.z_z[:] = 0.0   # w = 1*(1-0) = 1
    f.s_q[5, 2] = 3                                   # row 5, columns 16..23 -> w = 3
    W = orc.reconstruct(f)
    exp = np.ones((32, 32)); exp[5, 16:24] = 3.0
    assert np.array_equal(W, exp)
    f.s_q[5, 2] = 1
    f.s_s[1, 3] = 2.0                                 # tile rows 16..31, cols 24..31 -> w = 2
    exp = np.ones((32, 32)); exp[16:32, 24:32] = 2.0
    assert np.array_equal(orc.reconstruct(f), exp)
    # axis 1: group = rows [8r, 8r+8), column j; tile = 8 rows x 16 cols.
    g = tiny(32, 32, beta1=8, beta2=16, group_axis=1, outlier_rate=0.0)
    g.Q[:] = 1; g.s_q[:] = 1; g.z_q[:] = 0
    g.s_s[:] = 1.0; g.z_s[:] = 0.0; g.s_z[:] = 1.0; g.z_z[:] = 0.0
    g.z_q[2, 5] = 3                                   # rows 16..23, column 5 -> w = 1*(1-3) = -2
    exp = np.ones((32, 32)); exp[16:24, 5] = -2.0
    assert np.array_equal(orc.reconstruct(g), exp)
    g.z_q[2, 5] = 0
    g.s_s[3, 1] = 2.0                                 # tile rows 24..31, cols 16..31
    exp = np.ones((32, 32)); exp[24:32, 16:32] = 2.0
    assert np.array_equal(orc.reconstruct(g), exp)


@pytest.mark.parametrize("w_bits,beta1,beta2,axis", [
    (3, 16, 16, 0), (3, 16, 16, 1), (4, 16, 16, 0), (4, 16, 16, 1),
    (3, 8, 32, 0), (3, 8, 32, 1), (2, 4, 8, 0), (8, 32, 4, 1),
])
def test_vectorised_equals_brute_force(w_bits, beta1, beta2, axis):
    tr, tc = synth.tile_shape(beta1, beta2, axis)
    m, n = 2 * tr, 3 * tc
    f = synth.make_matrix(m, n, w_bits=w_bits, beta1=beta1, beta2=beta2, group_axis=axis,
                          outlier_rate=0.05, seed=(11, w_bits, beta1, beta2, axis))
    Wb = np.array(brute.reconstruct(f))
    W = orc.reconstruct(f)
    assert np.allclose(W, Wb, rtol=1e-14, atol=1e-14)
    x = synth.make_x(n, 1, seed=(3,))[0]
    yb = np.array(brute.matvec(f, x))
    y = orc.matvec(f, x)[0]
    assert np.allclose(y, yb, rtol=1e-12, atol=1e-12)
    rows = np.array([0, m // 2, m - 1])
    assert np.allclose(orc.matvec_rows(f, x, rows)[0], yb[rows], rtol=1e-12, atol=1e-12)


def test_exact_rational_arithmetic_single_weights():
    # fp16 inputs are exact rationals: evaluate s_s*(s_q - z_s) * (q - s_z*(z_q - z_z))
    # in exact arithmetic and compare (binary64 carries at most a few ulp of error).
    f = tiny(32, 48, w_bits=4, beta1=16, beta2=16, group_axis=1, outlier_rate=0.0)
    W = orc.reconstruct(f)
    for (i, j) in [(0, 0), (17, 5), (31, 47), (16, 31), (15, 32)]:
        ti, tj = i // 16, j // 16
        fr = lambda a: Fraction(float(a))
        s_hat = fr(f.s_s[ti, tj]) * (int(f.s_q[i // 16, j]) - fr(f.z_s[ti, tj]))
        z_hat = fr(f.s_z[ti, tj]) * (int(f.z_q[i // 16, j]) - fr(f.z_z[ti, tj]))
        exact = float(s_hat * (int(f.Q[i, j]) - z_hat))
        assert abs(W[i, j] - exact) <= 4 * np.spacing(abs(exact))


# ---- P2: Q = 0 and z_hat = 0  =>  only the outlier SpMV (library routine) -----
@pytest.mark.parametrize("axis", [0, 1])
def test_zero_codes_zero_zero_point_is_pure_spmv(axis):
    f = tiny(64, 96, group_axis=axis, outlier_rate=0.03)
    f.Q[:] = 0
    f.z_q[:] = 0; f.z_z[:] = 0.0          # z_hat = s_z*(0-0) = 0
    x = synth.make_x(96, 2, seed=(5,))
    S = sp.csr_matrix((f.val.astype(np.float64), f.col_idx.astype(np.int64),
                       f.row_ptr.astype(np.int64)), shape=(64, 96))
    ref = (S @ x.astype(np.float64).T).T
    assert np.allclose(orc.matvec(f, x), ref, rtol=1e-13, atol=1e-13)
    # zero second-level scale of the scales also kills the dense part
    g = tiny(64, 96, group_axis=axis, outlier_rate=0.03)
    g.s_s[:] = 0.0
    S = sp.csr_matrix((g.val.astype(np.float64), g.col_idx.astype(np.int64),
                       g.row_ptr.astype(np.int64)), shape=(64, 96))
    assert np.allclose(orc.matvec(g, x), (S @ x.astype(np.float64).T).T, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("axis", [0, 1])
def test_zero_codes_nonzero_zero_point_closed_form(axis):
    # Q = 0 => W = -s_hat*z_hat, so y_i = -sum_g s_hat_g z_hat_g sum_{j in g} x_j.
    f = tiny(32, 64, group_axis=axis, outlier_rate=0.0)
    f.Q[:] = 0
    # constant statistics everywhere: s_hat = 0.5*(3-1) = 1, z_hat = 0.25*(6-2) = 1
    f.s_q[:] = 3; f.z_q[:] = 6
    f.s_s[:] = 0.5; f.z_s[:] = 1.0; f.s_z[:] = 0.25; f.z_z[:] = 2.0
    x = synth.make_x(64, 1, seed=(6,))
    y = orc.matvec(f, x)[0]
    assert np.allclose(y, -x.astype(np.float64).sum(), rtol=1e-13)


# ---- P3: one-hot x extracts one column ----------------------------------------
@pytest.mark.parametrize("axis", [0, 1])
def test_one_hot_extracts_column(axis):
    f = tiny(48, 64, w_bits=4, group_axis=axis, outlier_rate=0.05)
    Wb = np.array(brute.reconstruct(f))
    for j in (0, 17, 63):
        e = np.zeros(64, dtype=np.float16); e[j] = 1.0
        assert np.allclose(orc.matvec(f, e)[0], Wb[:, j], rtol=1e-14, atol=1e-14)


# ---- P4: outlier-free, uniform statistics => integer matmul (textbook affine) --
@pytest.mark.parametrize("axis", [0, 1])
def test_uniform_stats_reduce_to_affine_integer_matmul(axis):
    f = tiny(64, 64, group_axis=axis, outlier_rate=0.0)
    f.s_q[:] = 5; f.z_q[:] = 7
    f.s_s[:] = 0.125; f.z_s[:] = 3.0      # s_hat = 0.125*2 = 0.25
    f.s_z[:] = 0.5; f.z_z[:] = 2.0        # z_hat = 0.5*5 = 2.5
    x = synth.make_x(64, 3, seed=(8,)).astype(np.float64)
    ref = 0.25 * (x @ f.Q.astype(np.float64).T - 2.5 * x.sum(axis=1, keepdims=True))
    assert np.allclose(orc.matvec(f, x.astype(np.float16)), ref, rtol=1e-12, atol=1e-12)


def test_per_group_scale_is_diagonal_scaling():
    # axis 1 with one row block (m = beta1): W = Q * s_hat[None, :] - (s_hat*z_hat)[None, :],
    # so y = Q @ (s_hat * x) - sum(s_hat*z_hat*x): a column scaling, via library matmul.
    f = tiny(16, 64, group_axis=1, outlier_rate=0.0)
    s_s = np.repeat(f.s_s[0].astype(np.float64), 16); z_s = np.repeat(f.z_s[0].astype(np.float64), 16)
    s_z = np.repeat(f.s_z[0].astype(np.float64), 16); z_z = np.repeat(f.z_z[0].astype(np.float64), 16)
    s_hat = s_s * (f.s_q[0] - z_s)
    z_hat = s_z * (f.z_q[0] - z_z)
    x = synth.make_x(64, 1, seed=(9,))[0].astype(np.float64)
    ref = f.Q.astype(np.float64) @ (s_hat * x) - np.sum(s_hat * z_hat * x)
    assert np.allclose(orc.matvec(f, x.astype(np.float16))[0], ref, rtol=1e-12, atol=1e-12)
    # axis 0 with one column block (n = beta1): a row scaling.
    g = tiny(64, 16, group_axis=0, outlier_rate=0.0)
    s_s = np.repeat(g.s_s[:, 0].astype(np.float64), 16); z_s = np.repeat(g.z_s[:, 0].astype(np.float64), 16)
    s_z = np.repeat(g.s_z[:, 0].astype(np.float64), 16); z_z = np.repeat(g.z_z[:, 0].astype(np.float64), 16)
    s_hat = s_s * (g.s_q[:, 0] - z_s)
    z_hat = s_z * (g.z_q[:, 0] - z_z)
    x = synth.make_x(16, 1, seed=(10,))[0].astype(np.float64)
    ref = s_hat * (g.Q.astype(np.float64) @ x - z_hat * x.sum())
    assert np.allclose(orc.matvec(g, x.astype(np.float16))[0], ref, rtol=1e-12, atol=1e-12)


def test_axis_swap_is_transpose():
    # Grouping along rows of W is grouping along columns of W^T.
    f = tiny(32, 64, beta1=8, beta2=16, group_axis=1, outlier_rate=0.0)
    ft = synth.SpQRLogical(f.n, f.m, f.w_bits, f.s_bits, f.z_bits, f.beta1, f.beta2, 0,
                           f.Q.T.copy(), f.s_q.T.copy(), f.z_q.T.copy(),
                           f.s_s.T.copy(), f.z_s.T.copy(), f.s_z.T.copy(), f.z_z.T.copy(),
                           np.zeros(f.n + 1, np.int32), f.col_idx[:0], f.val[:0])
    assert np.array_equal(orc.decode_dense(f), orc.decode_dense(ft).T)


# ---- P5 (oracle part): the size model reproduces the printed grid -------------
def test_average_bits_printed_grid():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "avg_bits_grid.txt"))
            if l.strip() and not l.startswith("#")]
    beta2s = [int(v) for v in rows[0][1:]]
    for r in rows[1:]:
        b1 = int(r[0])
        for b2, printed in zip(beta2s, r[1:]):
            dec = len(printed.split(".")[1]) if "." in printed else 0
            got = orc.average_bits(3, 3, 3, b1, b2)
            assert abs(got - float(printed)) <= 0.5 * 10 ** -dec + 1e-12, (b1, b2, got, printed)


def test_average_bits_printed_examples():
    for l in open(os.path.join(GOLDEN, "avg_bits_examples.txt")):
        if not l.strip() or l.startswith("#"):
            continue
        bw, bs, bz, b1, b2, ro, printed, dec = l.split()
        got = orc.average_bits(int(bw), int(bs), int(bz), int(b1), int(b2), float(ro))
        assert abs(got - float(printed)) <= 0.5 * 10 ** -int(dec) + 1e-12


# ---- P6 / P7: linearity and dense + sparse split -------------------------------
@pytest.mark.parametrize("axis", [0, 1])
def test_linearity_and_split(axis):
    f = tiny(64, 128, group_axis=axis, outlier_rate=0.02)
    x1 = synth.make_x(128, 1, seed=(1,)); x2 = synth.make_x(128, 1, seed=(2,))
    y1 = orc.matvec(f, x1); y2 = orc.matvec(f, x2)
    assert np.array_equal(orc.matvec(f, (x1 * np.float16(4.0))), 4.0 * y1)   # power of two: exact
    ys = orc.matvec(f, x1.astype(np.float64) + x2.astype(np.float64))
    assert np.allclose(ys, y1 + y2, rtol=1e-12, atol=1e-12)
    assert np.allclose(orc.matvec_dense_only(f, x1) + orc.matvec_sparse_only(f, x1), y1,
                       rtol=1e-12, atol=1e-12)


def test_outliers_add_to_the_in_place_code():
    # The code under an outlier stays in place and the 16-bit value is added on top.
    f = tiny(16, 16, outlier_rate=0.0)
    dense = orc.decode_dense(f)
    f.row_ptr = np.zeros(17, np.int32); f.row_ptr[4:] = 1
    f.col_idx = np.array([9], np.uint16); f.val = np.array([0.75], np.float16)
    W = orc.reconstruct(f)
    exp = dense.copy(); exp[3, 9] += 0.75
    assert np.array_equal(W, exp)


# ---- P8: the per-group factoring identity --------------------------------------
def test_group_factoring_identity():
    f = tiny(32, 64, group_axis=0, outlier_rate=0.0)
    s_hat, z_hat = orc.decode_stats(f)
    x = synth.make_x(64, 1, seed=(4,))[0].astype(np.float64)
    xg = x.reshape(-1, 16)
    qx = np.einsum("igk,gk->ig", f.Q.reshape(32, -1, 16).astype(np.float64), xg)
    y = np.sum(s_hat * (qx - z_hat * xg.sum(axis=1)[None, :]), axis=1)
    assert np.allclose(orc.matvec(f, x.astype(np.float16))[0], y, rtol=1e-12, atol=1e-12)


# ---- P9: sign conventions against the paper's encoder primitives ---------------
@pytest.mark.parametrize("bits", [3, 4])
def test_decoder_inverts_min_max_quantiser(bits):
    rng = np.random.default_rng(123)
    for _ in range(20):
        v = rng.normal(size=16) + rng.normal()        # groups need not straddle zero
        s, z = enc.fit_quantizer(v, bits)
        q = enc.quantize(v, s, z)
        assert q.min() == 0 and q.max() == 2 ** bits - 1
        assert q[np.argmin(v)] == 0 and q[np.argmax(v)] == 2 ** bits - 1
        back = orc.dequantize(q, s, z)
        assert np.max(np.abs(back - v)) <= s / 2 + 1e-12
        assert abs(back[np.argmin(v)] - v.min()) < 1e-12
        assert abs(back[np.argmax(v)] - v.max()) < 1e-12


def test_bilevel_roundtrip_through_encoder_primitives():
    # Quantise real group statistics with the second-level quantiser and check
    # the oracle's decoded statistics against them (error <= half a second-level step).
    rng = np.random.default_rng(5)
    f = tiny(16, 16, group_axis=0, outlier_rate=0.0)
    s_true = rng.uniform(0.01, 0.1, size=16); z_true = rng.uniform(1.0, 6.0, size=16)
    s_s, z_s = enc.fit_quantizer(s_true, 3); s_z, z_z = enc.fit_quantizer(z_true, 3)
    f.s_q[:, 0] = enc.quantize(s_true, s_s, z_s).astype(np.uint8)
    f.z_q[:, 0] = enc.quantize(z_true, s_z, z_z).astype(np.uint8)
    f.s_s[:] = s_s; f.z_s[:] = z_s; f.s_z[:] = s_z; f.z_z[:] = z_z
    s_hat, z_hat = orc.decode_stats(f)
    h = lambda a: float(np.float16(a))
    # fp16 storage of the four scalars perturbs the bound slightly
    assert np.max(np.abs(s_hat[:, 0] - s_true)) <= h(s_s) / 2 + 8 * 2e-3 * h(s_s) * 7 + 1e-6
    assert np.max(np.abs(z_hat[:, 0] - z_true)) <= h(s_z) / 2 + 8 * 2e-3 * h(s_z) * 7 + 1e-3


# ---- fp32 statistic path agrees with fp64 --------------------------------------
def test_f32_statistics_close_to_f64():
    f = tiny(64, 64, outlier_rate=0.0)
    s32, z32 = orc.decode_stats_f32(f)
    s64, z64 = orc.decode_stats(f)
    assert s32.dtype == np.float32
    assert np.allclose(s32, s64, rtol=2.0 ** -22, atol=0)
    assert np.allclose(z32, z64, rtol=2.0 ** -22, atol=0)


# ---- the generator itself ------------------------------------------------------
@pytest.mark.parametrize("structure", ["uniform", "rows8cols4", "cols64", "zipf"])
def test_generator_csr_is_valid(structure):
    f = synth.make_matrix(256, 512, outlier_rate=0.02, outlier_structure=structure, seed=(1, 2))
    budget = round(0.02 * 256 * 512)
    assert f.row_ptr[0] == 0 and f.row_ptr[-1] == f.nnz
    # the structured lines alone may exceed a small matrix's budget
    assert f.nnz == budget if structure in ("uniform", "zipf") else f.nnz >= budget
    assert np.all(np.diff(f.row_ptr) >= 0)
    for i in range(256):
        c = f.col_idx[f.row_ptr[i]:f.row_ptr[i + 1]].astype(np.int64)
        assert np.all(np.diff(c) > 0) and (c.size == 0 or c.max() < 512)
    counts = np.diff(f.row_ptr)
    if structure == "rows8cols4":
        assert np.sum(counts == 512) == 8
    if structure == "zipf":
        assert counts.max() == 512 and np.median(counts) < counts.mean()
    g = synth.make_matrix(256, 512, outlier_rate=0.02, outlier_structure=structure, seed=(1, 2))
    assert np.array_equal(f.Q, g.Q) and np.array_equal(f.col_idx, g.col_idx)


# ---- act-order input permutation (Sec. 5 ablations, App. B `permutation_order act_order`) -------
# An act-order quantiser reorders the INPUT dimension before the column sweep of Alg. 1 and stores
# the matrix in that order: stored column j is column perm[j] of the original weight.  The product
# with the original activations is  y = sum_j W_stored[:, j] * x[perm[j]].
def test_permutation_hand_case_three_cycle():
    f = tiny(16, 16, group_axis=0, outlier_rate=0.0)
    W = orc.reconstruct(f)                      # stored column order
    perm = np.arange(16, dtype=np.int32)
    perm[[2, 5, 11]] = [5, 11, 2]               # a 3-cycle: stored column 2 <- x[5], 5 <- x[11], 11 <- x[2]
    f.perm = perm
    k = 5
    x = np.zeros(16, dtype=np.float16); x[k] = 1.0
    y = orc.matvec(f, x)[0]
    j = int(np.nonzero(perm == k)[0][0])        # the stored column that meets x[k]: perm[j] = k -> j = 2
    assert j == 2 and perm[k] == 11
    assert np.array_equal(y, W[:, j])           # column j with perm[j] = k ...
    assert not np.array_equal(y, W[:, perm[k]])  # ... and NOT column perm[k] (the inverse reading)
    assert np.array_equal(orc.matvec_rows(f, x, np.arange(16))[0], W[:, j])
    assert np.array_equal(np.array(brute.matvec(f, x)), W[:, j])


@pytest.mark.parametrize("axis", [0, 1])
def test_permutation_equals_unpermuting_the_stored_matrix(axis):
    # Definition, independent of the oracle's own gather: scatter the stored columns back to the original
    # order (W_orig[:, perm[j]] = W_stored[:, j]) and multiply by x as it is.
    f = tiny(32, 48, group_axis=axis, outlier_rate=0.04)
    rng = np.random.default_rng(21)
    perm = rng.permutation(48).astype(np.int32)
    Ws = orc.reconstruct(f)
    W_orig = np.empty_like(Ws)
    for j in range(48):
        W_orig[:, perm[j]] = Ws[:, j]
    X = synth.make_x(48, 3, seed=(22,))
    ref = X.astype(np.float64) @ W_orig.T
    f.perm = perm
    assert np.allclose(orc.matvec(f, X), ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(orc.matvec_dense_only(f, X) + orc.matvec_sparse_only(f, X), ref, rtol=1e-12, atol=1e-12)
    rows = np.array([0, 7, 31])
    assert np.allclose(orc.matvec_rows(f, X, rows), ref[:, rows], rtol=1e-12, atol=1e-12)
    for b in range(3):
        assert np.allclose(np.array(brute.matvec(f, X[b])), ref[b], rtol=1e-12, atol=1e-12)


def test_identity_permutation_is_a_no_op():
    f = tiny(32, 32, outlier_rate=0.05)
    X = synth.make_x(32, 2, seed=(23,))
    ref = orc.matvec(f, X)
    f.perm = np.arange(32, dtype=np.int32)
    assert np.allclose(orc.matvec(f, X), ref, rtol=1e-14, atol=1e-14)   # a gathered copy may be summed in another order
    assert np.array_equal(np.array(brute.matvec(f, X[0])), np.array(brute.matvec(
        synth.SpQRLogical(**{**f.__dict__, "perm": None}), X[0])))


# ---- statistic variants of the ablations (Sec. 5): integer zero-point, 16-bit statistics ----
def _variant(m, n, layout, **kw):
    kw.setdefault("seed", (13, m, n))
    return synth.make_matrix(m, n, stat_layout=layout, **kw)


def test_round_zero_hand_values():
    # s_s = 0.5, z_s = 1, s_q = 3 -> s_hat = 1; zero-point = the code itself
    for axis in (0, 1):
        f = _variant(16, 16, "round_zero", group_axis=axis, outlier_rate=0.0)
        assert f.s_z is None and f.z_z is None
        f.Q[:] = 5; f.s_q[:] = 3; f.z_q[:] = 4
        f.s_s[:] = 0.5; f.z_s[:] = 1.0
        assert np.all(orc.reconstruct(f) == 1.0)          # 1 * (5 - 4)
        f.z_q[:] = 7
        assert np.all(orc.reconstruct(f) == -2.0)         # 1 * (5 - 7)
        f.z_s[:] = 2.0
        assert np.all(orc.reconstruct(f) == -1.0)         # 0.5 * (5 - 7)
    # one group's zero code moves exactly that group (axis 1: rows [8r, 8r+8) of column j)
    g = _variant(32, 32, "round_zero", beta1=8, beta2=16, group_axis=1, outlier_rate=0.0)
    g.Q[:] = 1; g.s_q[:] = 1; g.z_q[:] = 0; g.s_s[:] = 1.0; g.z_s[:] = 0.0
    g.z_q[2, 5] = 3
    exp = np.ones((32, 32)); exp[16:24, 5] = -2.0
    assert np.array_equal(orc.reconstruct(g), exp)


@pytest.mark.parametrize("axis", [0, 1])
def test_round_zero_is_bilevel_with_a_unit_zero_quantiser(axis):
    # An integer zero-point is what the (already pinned) bilevel decode gives for s_z = 1, z_z = 0.
    f = _variant(64, 96, "round_zero", w_bits=3, beta1=8, beta2=32, group_axis=axis, outlier_rate=0.03)
    b = synth.make_matrix(64, 96, w_bits=3, beta1=8, beta2=32, group_axis=axis, outlier_rate=0.03,
                          seed=(13, 64, 96))
    assert np.array_equal(b.Q, f.Q) and np.array_equal(b.s_q, f.s_q) and np.array_equal(b.s_s, f.s_s)
    b.s_z[:] = 1.0; b.z_z[:] = 0.0
    assert np.array_equal(orc.reconstruct(f), orc.reconstruct(b))
    x = synth.make_x(96, 2, seed=(5,))
    assert np.array_equal(orc.matvec(f, x), orc.matvec(b, x))
    # and it is not the bilevel decode of the drawn (s_z, z_z)
    assert not np.allclose(orc.reconstruct(f), orc.reconstruct(
        synth.make_matrix(64, 96, w_bits=3, beta1=8, beta2=32, group_axis=axis, outlier_rate=0.03, seed=(13, 64, 96))))


def test_stats16_hand_values():
    for axis in (0, 1):
        f = _variant(16, 16, "stats16", group_axis=axis, outlier_rate=0.0)
        assert f.s_q is None and f.s_s is None and f.s16.dtype == np.float16
        f.Q[:] = 5; f.s16[:] = 0.5; f.z16[:] = 1.5
        assert np.all(orc.reconstruct(f) == 1.75)         # 0.5 * (5 - 1.5)
    # group indexing: axis 0, group = row i, columns [8c, 8c+8)
    f = _variant(32, 32, "stats16", beta1=8, beta2=16, group_axis=0, outlier_rate=0.0)
    f.Q[:] = 2; f.s16[:] = 1.0; f.z16[:] = 0.0
    f.s16[5, 2] = 3.0
    exp = np.full((32, 32), 2.0); exp[5, 16:24] = 6.0
    assert np.array_equal(orc.reconstruct(f), exp)
    f.s16[5, 2] = 1.0; f.z16[30, 0] = 0.5
    exp = np.full((32, 32), 2.0); exp[30, 0:8] = 1.5
    assert np.array_equal(orc.reconstruct(f), exp)
    # axis 1, group = rows [8r, 8r+8) of column j
    g = _variant(32, 32, "stats16", beta1=8, beta2=16, group_axis=1, outlier_rate=0.0)
    g.Q[:] = 2; g.s16[:] = 1.0; g.z16[:] = 0.0
    g.z16[1, 31] = 4.0
    exp = np.full((32, 32), 2.0); exp[8:16, 31] = -2.0
    assert np.array_equal(orc.reconstruct(g), exp)


@pytest.mark.parametrize("axis", [0, 1])
def test_stats16_equals_bilevel_whose_statistics_are_16_bit_numbers(axis):
    # A bilevel matrix with s_s = 0.5, z_s = 1, s_z = 0.25, z_z = 2 decodes to statistics that are exact 16-bit
    # floats; storing those directly must give the same matrix.
    b = synth.make_matrix(48, 64, w_bits=4, beta1=16, beta2=16, group_axis=axis, outlier_rate=0.02, seed=(17,))
    b.s_s[:] = 0.5; b.z_s[:] = 1.0; b.s_z[:] = 0.25; b.z_z[:] = 2.0
    f = _variant(48, 64, "stats16", w_bits=4, beta1=16, beta2=16, group_axis=axis, outlier_rate=0.02, seed=(17,))
    f.Q = b.Q; f.row_ptr, f.col_idx, f.val = b.row_ptr, b.col_idx, b.val
    f.s16 = (0.5 * (b.s_q.astype(np.float64) - 1.0)).astype(np.float16)
    f.z16 = (0.25 * (b.z_q.astype(np.float64) - 2.0)).astype(np.float16)
    assert np.array_equal(orc.reconstruct(f), orc.reconstruct(b))


@pytest.mark.parametrize("layout,w_bits,beta1,beta2,axis", [
    ("round_zero", 3, 16, 16, 0), ("round_zero", 3, 8, 32, 1), ("round_zero", 4, 16, 16, 1),
    ("stats16", 3, 16, 16, 0), ("stats16", 3, 48, 16, 1), ("stats16", 4, 8, 32, 0),
])
def test_variants_vectorised_equals_brute_force(layout, w_bits, beta1, beta2, axis):
    tr, tc = synth.tile_shape(beta1, beta2, axis)
    m, n = 2 * tr, 3 * tc
    f = synth.make_matrix(m, n, w_bits=w_bits, beta1=beta1, beta2=beta2, group_axis=axis, outlier_rate=0.05,
                          seed=(19, w_bits, beta1, beta2, axis), stat_layout=layout)
    assert np.allclose(orc.reconstruct(f), np.array(brute.reconstruct(f)), rtol=1e-14, atol=1e-14)
    x = synth.make_x(n, 1, seed=(3,))[0]
    yb = np.array(brute.matvec(f, x))
    assert np.allclose(orc.matvec(f, x)[0], yb, rtol=1e-12, atol=1e-12)
    rows = np.array([0, m // 2, m - 1])
    assert np.allclose(orc.matvec_rows(f, x, rows)[0], yb[rows], rtol=1e-12, atol=1e-12)
    s32, z32 = orc.decode_stats_f32(f)
    s64, z64 = orc.decode_stats(f)
    assert np.allclose(s32, s64, rtol=1e-6) and np.allclose(z32, z64, rtol=1e-6, atol=1e-7)


def test_stats16_inverts_the_min_max_quantiser():
    # Alg. 1 without the second level: fit (s, z) per group of 16 weights, keep them as 16-bit floats,
    # quantise with them; the decode is within half a step of every weight.
    rng = np.random.default_rng(23)
    f = _variant(16, 64, "stats16", w_bits=3, beta1=16, beta2=16, group_axis=0, outlier_rate=0.0)
    W = rng.standard_normal((16, 64))
    for i in range(16):
        for c in range(4):
            grp = W[i, 16 * c:16 * c + 16]
            s, z = enc.fit_quantizer(grp, 3)
            f.s16[i, c] = s; f.z16[i, c] = z
            s16, z16 = float(f.s16[i, c]), float(f.z16[i, c])
            f.Q[i, 16 * c:16 * c + 16] = np.clip(enc.quantize(grp, s16, z16), 0, 7)
    err = np.abs(orc.reconstruct(f) - W)
    step = np.repeat(f.s16.astype(np.float64), 16, axis=1)
    # codes clipped at the range's ends can be off by the rounding of (s, z) to 16 bit: a little over half a step
    assert np.all(err <= 0.5 * step * 1.02 + 1e-3)
    assert np.max(err) > 0.2 * step.min()


def test_average_bits_of_the_variants_printed_values():
    path = os.path.join(os.path.dirname(__file__), "golden", "avg_bits_ablation.txt")
    seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        lay, b_w, b1, b2, printed, dec = line.split()
        b_w, b1, b2, printed, dec = int(b_w), int(b1), int(b2), float(printed), int(dec)
        if lay == "stats16":
            v = orc.average_bits_stats16(b_w, b1)
        else:
            v = orc.average_bits(b_w, 3, 3, b1, b2)
        assert abs(v - printed) <= 0.5 * 10 ** -dec + 1e-12, (lay, v, printed)
        seen += 1
    assert seen == 3
    # one second-level pair less per tile of beta1*beta2 weights
    assert orc.average_bits(3, 3, 3, 16, 16) - orc.average_bits_round_zero(3, 3, 3, 16, 16) == 32.0 / 256.0
    assert orc.average_bits_round_zero(3, 3, 3, 16, 16) == 3.5
    assert orc.average_bits_stats16(3, 16) == 5.0
