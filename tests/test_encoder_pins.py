"""CPU pins of the quantiser oracle (oracle/spqr_encoder.py, Alg. 1): what the paper and the mathematics fix.

  * H^ic: the defining identity U^T U (H + lambda I) = I, triangularity, the closed form for a diagonal H;
  * the error-feedback sweep: the optimal-brain-surgeon identity  delta (H + lambda I) delta^T = sum_j E_j^2  per
    row (delta = W - W_final), which a wrong sign, index, transposed H^ic or a missing 1 / H^ic_jj breaks;
  * H^ic = I: the sweep degenerates to round-to-nearest with bilevel statistics, checked weight by weight;
  * subroutines: code 0 <-> min, 2^b - 1 <-> max, error <= s / 2 (Alg. 1 fit_quantizer / quantize / dequantize);
  * the outlier test on a hand-made group, and App. B's statement that raising tau never adds outliers;
  * what the decoder oracle reconstructs from the encoder's output is the matrix the sweep left (codes, both
    statistic levels, CSR order and the additive outlier values agree with Sec. 4.2's format);
  * the whole procedure against scalar pure-Python loops on tiny matrices, bit for bit.
"""
import numpy as np
import pytest

from oracle import brute_encoder, spqr_encoder as enc, spqr_oracle as orc


def _problem(seed, m, n, d=None, corr=0.3, heavy=0.02):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.05, (m, n))
    W[rng.random((m, n)) < heavy] *= 6.0
    A = rng.normal(size=(n, n)) * corr + np.eye(n)
    X = A @ rng.normal(size=(n, d or 4 * n))
    return W, X


def test_inverse_cholesky_identity_and_closed_form():
    W, X = _problem(1, 8, 48)
    H = enc.hessian(X)
    assert np.allclose(H, 2 * X @ X.T) and np.allclose(H, H.T)
    lam = 0.5
    U = enc.inverse_cholesky(H, lam)
    assert np.array_equal(U, np.triu(U)) and (np.diagonal(U) > 0).all()
    assert np.abs(U.T @ U @ (H + lam * np.eye(48)) - np.eye(48)).max() < 1e-10
    # a row of U right of the diagonal is not a column: U U^T is NOT the inverse for a correlated H
    assert np.abs(U @ U.T @ (H + lam * np.eye(48)) - np.eye(48)).max() > 1e-3
    d = np.array([1.0, 4.0, 9.0, 16.0])
    assert np.allclose(enc.inverse_cholesky(np.diag(d), 0.0), np.diag(1.0 / np.sqrt(d)))
    assert np.allclose(enc.inverse_cholesky(np.diag(d), 3.0), np.diag(1.0 / np.sqrt(d + 3.0)))


def test_quantizer_primitives():
    rng = np.random.default_rng(2)
    for bits in (2, 3, 4):
        M = rng.normal(size=(50, 16)) + rng.normal(size=(50, 1)) * 3      # all-positive and all-negative groups too
        s, z = enc.fit_quantizer(M, bits)
        q = enc.quantize(M, s[:, None], z[:, None], bits)
        assert q.min() == 0 and q.max() == 2 ** bits - 1
        assert (q[np.arange(50), M.argmin(1)] == 0).all() and (q[np.arange(50), M.argmax(1)] == 2 ** bits - 1).all()
        back = enc.dequantize(q, s[:, None], z[:, None])
        assert (np.abs(back - M) <= s[:, None] / 2 * (1 + 1e-9)).all()
    # hand values: group {1, 2, 4}, 2 bits: s = 1, z = -1; 2.4 -> code 1, 2.6 -> code 2 (round half up: 2.5 -> 2)
    s, z = enc.fit_quantizer(np.array([[1.0, 2.0, 4.0]]), 2)
    assert s[0] == 1.0 and z[0] == -1.0
    assert list(enc.quantize(np.array([2.4, 2.6, 2.5, -7.0, 99.0]), 1.0, -1.0, 2)) == [1, 2, 2, 0, 3]
    # flat group: exact
    s, z = enc.fit_quantizer(np.array([[0.3, 0.3]]), 3)
    assert enc.dequantize(enc.quantize(0.3, s, z, 3), s, z)[0] == 0.3
    # masked fit leaves the outlier out of the range instead of replacing it by zero
    s, z = enc.fit_quantizer(np.array([[1.0, 2.0, 50.0]]), 3, keep=np.array([[True, True, False]]))
    assert s[0] == 1.0 / 7 and z[0] == -7.0


def test_outlier_test_by_hand_and_monotone_in_tau():
    # group {0, 1, 2, 3, 4, 5, 6, 100}, 3 bits, H^ic diagonal 1: fitted on all eight the step is 100/7, every small
    # weight rounds to 0 (error w^2): base = 1+4+9+16+25+36 = 91.  Without the 100 the seven others are exact: the
    # reduction is 91.  Without the weight 6 nothing improves except its own error 36; without the weight 0 the range
    # starts at 1 and the others' errors become (w - 1)^2: 55, a reduction of 36 as well; without the weight 3: 9.
    Wb = np.array([[0.0, 1, 2, 3, 4, 5, 6, 100]])
    hd = np.ones(8)
    assert enc.error(Wb, hd, 3).sum() == pytest.approx(91.0, abs=1e-9)
    assert list(enc.outliers(Wb, hd, 3, 90.0)[0]) == [False] * 7 + [True]
    assert list(enc.outliers(Wb, hd, 3, 92.0)[0]) == [False] * 8
    assert list(enc.outliers(Wb, hd, 3, 35.0)[0]) == [True] + [False] * 5 + [True, True]
    assert list(enc.outliers(Wb, hd, 3, 36.5)[0]) == [False] * 7 + [True]
    assert list(enc.outliers(Wb, hd, 3, 8.5)[0]) == [True, False, False, True, True, True, True, True]
    # the error is measured in units of H^ic_jj: halving the diagonal quadruples it
    assert enc.error(Wb, 0.5 * hd, 3).sum() == pytest.approx(4 * 91.0, abs=1e-9)
    # App. B: for a fixed configuration a larger tau never gives more outliers
    W, X = _problem(3, 32, 64)
    U = enc.inverse_cholesky(enc.hessian(X), 0.1)
    counts = [int(enc.spqr_quantize(W, U, 3, 16, 16, tau).row_ptr[-1]) for tau in (0.0, 0.05, 0.2, 1.0, 1e9)]
    assert counts == sorted(counts, reverse=True) and counts[-1] == 0 and counts[0] > counts[2] > 0


@pytest.mark.parametrize("bits,b1,b2,tau", [(3, 16, 16, 1e9), (3, 16, 16, 0.3), (4, 16, 16, 0.1), (3, 8, 32, 0.2)])
def test_sweep_satisfies_the_obs_identity(bits, b1, b2, tau):
    W, X = _problem(4, 64, 96)
    lam = 0.05
    H = enc.hessian(X)
    r = enc.spqr_quantize(W, enc.inverse_cholesky(H, lam), bits, b1, b2, tau)
    delta = W - r.W_final
    lhs = np.einsum("ij,jk,ik->i", delta, H + lam * np.eye(96), delta)
    rhs = (r.E ** 2).sum(axis=1)
    assert np.abs(lhs - rhs).max() <= 1e-9 * max(1.0, lhs.max())
    assert (r.E[r.is_outlier] == 0).all()
    if tau < 1e8:
        assert 0 < r.row_ptr[-1] < W.size // 2
    # the error feedback pays: output error below that of the same quantiser without it (H^ic = identity)
    rtn = enc.spqr_quantize(W, np.eye(96), bits, b1, b2, 1e9)
    if tau > 1e8:
        assert np.linalg.norm((W - r.W_final) @ X) < 0.9 * np.linalg.norm((W - rtn.W_final) @ X)


def test_identity_hessian_is_round_to_nearest_with_bilevel_statistics():
    W, _ = _problem(5, 32, 32)
    bits, b1, b2 = 3, 8, 16
    r = enc.spqr_quantize(W, np.eye(32), bits, b1, b2, 1e9)
    assert r.row_ptr[-1] == 0
    for t in range(32 // b2):
        for g in range(32 // b1):
            blk = W[t * b2:(t + 1) * b2, g * b1:(g + 1) * b1]
            lo, hi = blk.min(1), blk.max(1)
            s = (hi - lo) / 7.0
            z = -lo / s
            ss = np.float64(np.float16((s.max() - s.min()) / 7.0)); zs = np.float64(np.float16(-s.min() / ((s.max() - s.min()) / 7.0)))
            sz = np.float64(np.float16((z.max() - z.min()) / 7.0)); zz = np.float64(np.float16(-z.min() / ((z.max() - z.min()) / 7.0)))
            assert r.s_s[t, g] == ss and r.z_s[t, g] == zs and r.s_z[t, g] == sz and r.z_z[t, g] == zz
            sq = np.clip(np.floor(s / ss + zs + 0.5), 0, 7); zq = np.clip(np.floor(z / sz + zz + 0.5), 0, 7)
            assert (r.s_q[t * b2:(t + 1) * b2, g] == sq).all() and (r.z_q[t * b2:(t + 1) * b2, g] == zq).all()
            sh = ss * (sq - zs); zh = sz * (zq - zz)
            q = np.clip(np.floor(blk / sh[:, None] + zh[:, None] + 0.5), 0, 7)
            assert (r.Q[t * b2:(t + 1) * b2, g * b1:(g + 1) * b1] == q).all()
            # line 14 leaves W - ((W - w_q) / 1) * 1 in place of a quantised weight: w_q up to one rounding
            assert np.abs(r.W_final[t * b2:(t + 1) * b2, g * b1:(g + 1) * b1] - sh[:, None] * (q - zh[:, None])).max() < 1e-15


@pytest.mark.parametrize("bits,b1,b2,tau", [(3, 16, 16, 0.3), (4, 8, 32, 0.1)])
def test_decoder_oracle_reconstructs_what_the_sweep_left(bits, b1, b2, tau):
    W, X = _problem(6, 64, 64)
    r = enc.spqr_quantize_from_calibration(W, X, bits, b1, b2, tau, 0.05)
    assert r.group_axis == 0 and r.Q.max() <= 2 ** bits - 1 and r.s_q.max() <= 7 and r.z_q.max() <= 7
    dense = orc.decode_dense(r)
    base = ~r.is_outlier
    assert np.abs(dense - r.W_final)[base].max() < 1e-13           # line 14 leaves w_q up to a rounding or two
    full = orc.reconstruct(r)
    rows = np.repeat(np.arange(64), np.diff(r.row_ptr))
    assert r.is_outlier[rows, r.col_idx].all() and len(rows) == r.is_outlier.sum()
    for a in range(64):                                            # by row, then by column
        assert (np.diff(r.col_idx[r.row_ptr[a]:r.row_ptr[a + 1]].astype(int)) > 0).all()
    err = np.abs(full - r.W_final)[r.is_outlier]
    assert (err <= np.maximum(2.0 ** -11 * np.abs(r.val.astype(np.float64)), 2.0 ** -25) + 1e-12).all()   # half an ulp (subnormals: 2^-25)
    # size model of App. D with the outlier rate the sweep produced
    assert orc.average_bits(bits, 3, 3, b1, b2, r.row_ptr[-1] / W.size) == pytest.approx(
        bits + 6 / b1 + 64 / (b1 * b2) + 32 * r.row_ptr[-1] / W.size)


@pytest.mark.parametrize("bits,b1,b2,tau,m,n", [(3, 4, 4, 0.02, 8, 12), (2, 4, 2, 0.0005, 4, 8), (3, 8, 4, 1e9, 4, 16),
                                                (4, 4, 8, 0.001, 8, 8)])
def test_vectorised_equals_scalar_loops(bits, b1, b2, tau, m, n):
    W, X = _problem(7 + m + n, m, n, heavy=0.1)
    U = enc.inverse_cholesky(enc.hessian(X), 0.01)
    r = enc.spqr_quantize(W, U, bits, b1, b2, tau)
    b = brute_encoder.spqr_quantize(W, U, bits, b1, b2, tau)
    for k in ("Q", "s_q", "z_q", "s_s", "z_s", "s_z", "z_z", "row_ptr", "col_idx"):
        assert np.array_equal(np.asarray(getattr(r, k), dtype=np.float64), np.asarray(b[k], dtype=np.float64)), k
    assert np.array_equal(r.val, b["val"]) and np.array_equal(r.W_final, b["W_final"])
    if tau < 1:
        assert 0 < r.row_ptr[-1] < m * n


def test_act_order_reading_and_direction():
    # order: decreasing diagonal, ties to the smaller index
    H = np.diag([3.0, 7.0, 3.0, 9.0, 7.0])
    assert list(enc.act_order(H)) == [3, 1, 4, 0, 2]
    assert list(enc.act_order(np.diag([5.0, 4.0, 3.0]))) == [0, 1, 2]
    # direction: the stored matrix is W[:, perm] and meets x[perm[j]]: with 8-bit codes (error ~ 1e-3 of the weights) the
    # decoder oracle's product with `perm` reproduces W x; with the inverse permutation it does not
    W, X = _problem(8, 32, 48)
    X = X * np.linspace(0.5, 3.0, 48)[::-1, None] * np.where(np.arange(48) % 2, 1.0, 0.3)[:, None]   # distinct input scales
    r = enc.spqr_quantize_act_order(W, X, 8, 16, 16, 1e9, 0.01)
    assert sorted(r.perm) == list(range(48)) and list(r.perm) != list(range(48))
    d = np.diagonal(enc.hessian(X))[r.perm]
    assert (np.diff(d) <= 0).all()
    # (on a calibration input: the error feedback minimises the error on those, not on arbitrary vectors)
    x = (X[:, :1].T / np.abs(X).max()).astype(np.float16)
    want = W @ x[0].astype(np.float64)
    y = orc.matvec(r, x)[0]
    assert np.linalg.norm(y - want) <= 2e-2 * np.linalg.norm(want)
    inv = np.empty_like(r.perm); inv[r.perm] = np.arange(48)
    wrong = enc.spqr_quantize_act_order(W, X, 8, 16, 16, 1e9, 0.01); wrong.perm = inv
    assert np.linalg.norm(orc.matvec(wrong, x)[0] - want) > 0.3 * np.linalg.norm(want)
    # the sweep itself is Alg. 1 on the permuted problem
    H = enc.hessian(X)
    ref = enc.spqr_quantize(W[:, r.perm], enc.inverse_cholesky(H[np.ix_(r.perm, r.perm)], 0.01), 8, 16, 16, 1e9)
    assert np.array_equal(ref.Q, r.Q)
