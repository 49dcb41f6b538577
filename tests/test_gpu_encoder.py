"""GPU parity of the quantiser (Alg. 1, include/spqr_encode.h) against the CPU oracle (oracle/spqr_encoder.py).

Bars:
  * spqr_quantize (the sweep: outlier test, statistic fit, codes, error feedback, outlier values): BIT-EXACT against
    the oracle on the same W and H^ic - every integer output, the 16-bit statistics and outlier values, and the
    binary64 weights the sweep leaves.  Both sides take every decision in binary64, one rounded operation per step
    in the same order;
  * spqr_hessian, spqr_inverse_cholesky: floating-point linear algebra in another summation order than LAPACK's:
    relative 1e-11 on H, the defining identity H^ic^T H^ic (H + lambda I) = I to 1e-9 and 1e-8 relative to the
    oracle's factor (condition numbers of the test Hessians are ~1e3);
  * the whole chain on the GPU (its own H^ic): the output error ||(W - W_hat) X|| within 2 % of the oracle's chain,
    and the packed result multiplies like the decoder oracle says.
"""
import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_encoder as enc, spqr_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    import torch
    import paper_2306_03078_amd as P
    import paper_2306_03078_amd.encode_binding as E
    P.load_library()
    assert torch.cuda.is_available()
    return E


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


@pytest.mark.parametrize("n,d", [(64, 64), (96, 200), (200, 333), (256, 1024)])
def test_hessian(E, n, d):
    _, X = synth.make_quantizer_problem(1, 16, n, d)
    H = E.spqr_hessian(dev(X)).cpu().numpy()
    ref = enc.hessian(X)
    assert np.array_equal(H, H.T)
    assert np.abs(H - ref).max() <= 1e-11 * np.abs(ref).max()


@pytest.mark.parametrize("n,lam", [(64, 0.5), (96, 0.05), (200, 1.0), (256, 0.01), (640, 0.1), (1000, 0.1), (1472, 0.2)])
def test_inverse_cholesky(E, n, lam):
    _, X = synth.make_quantizer_problem(2, 16, n)
    H = enc.hessian(X)
    U = E.spqr_inverse_cholesky(dev(H), lam).cpu().numpy()
    assert np.array_equal(U, np.triu(U)) and (np.diagonal(U) > 0).all()
    assert np.abs(U.T @ U @ (H + lam * np.eye(n)) - np.eye(n)).max() < 1e-9
    ref = enc.inverse_cholesky(H, lam)
    assert np.abs(U - ref).max() <= 1e-8 * np.abs(ref).max()


def _compare_exact(got, ref):
    assert np.isfinite(ref.W_final).all()
    bad = [k for k in ("Q", "s_q", "z_q", "row_ptr", "col_idx")
           if not np.array_equal(np.asarray(getattr(got, k), dtype=np.int64), np.asarray(getattr(ref, k), dtype=np.int64))]
    bad += [k for k in ("s_s", "z_s", "s_z", "z_z", "val")
            if not np.array_equal(np.asarray(getattr(got, k)).view(np.uint16), np.asarray(getattr(ref, k)).view(np.uint16))]
    if not np.array_equal(got.is_outlier, ref.is_outlier):
        bad.append("is_outlier")
    if not np.array_equal(got.W_final.view(np.uint64), ref.W_final.view(np.uint64)):
        bad.append("W_final")
    assert not bad, bad


@pytest.mark.parametrize("bits,b1,b2,tau,m,n", [
    (3, 16, 16, 1.0, 128, 256), (4, 16, 16, 0.4, 64, 128), (3, 8, 32, 0.8, 96, 192), (3, 32, 16, 1.2, 80, 128),
    (3, 4, 4, 0.2, 68, 64), (2, 8, 2, 1.2, 6, 40), (3, 16, 64, 0.8, 192, 96), (3, 16, 16, float("inf"), 144, 160),
    (8, 8, 8, 1e-6, 72, 64)])
def test_sweep_is_bit_exact(E, bits, b1, b2, tau, m, n):
    W, X = synth.make_quantizer_problem(3 + m + n, m, n)
    U = enc.inverse_cholesky(enc.hessian(X), 0.05)
    ref = enc.spqr_quantize(W, U, bits, b1, b2, tau)
    got = E.spqr_quantize(dev(W), dev(U), bits, b1, b2, tau)
    _compare_exact(got, ref)
    if np.isfinite(tau):
        assert 0 < ref.row_ptr[-1] < m * n          # the case does have outliers, and not only outliers


def test_sweep_is_bit_exact_at_layer_size(E):
    # a 1024 x 1024 layer, 3-bit, beta1 = beta2 = 16: 64 column blocks, 16 workgroups, every wavefront's share of
    # the trailing columns several chunks long
    W, X = synth.make_quantizer_problem(11, 1024, 1024, 2048)
    U = enc.inverse_cholesky(enc.hessian(X), 0.1)
    ref = enc.spqr_quantize(W, U, 3, 16, 16, 3.0)
    got = E.spqr_quantize(dev(W), dev(U), 3, 16, 16, 3.0)
    _compare_exact(got, ref)
    rate = ref.row_ptr[-1] / W.size
    assert 0.001 < rate < 0.2


def test_degenerate_groups(E):
    # flat groups (max = min), a group whose weights are all outliers but one, zeros, and equal statistics in a tile
    rng = np.random.default_rng(5)
    m, n = 64, 64
    W = rng.normal(0, 0.05, (m, n))
    W[:16, :16] = 0.25            # a flat tile: s = 1, z = -0.25 everywhere, second level flat too
    W[16:32, 16:32] = 0.0
    W[40, 32:48] = np.linspace(-1, 1, 16) ** 3 * 5
    U = np.eye(n)
    for tau in (float("inf"), 1e-4):
        ref = enc.spqr_quantize(W, U, 3, 16, 16, tau)
        got = E.spqr_quantize(dev(W), dev(U), 3, 16, 16, tau)
        _compare_exact(got, ref)


def test_whole_chain_on_the_gpu(E):
    import torch
    import paper_2306_03078_amd as P
    m, n, bits, b1, b2, tau, lam = 256, 256, 3, 16, 16, 1.0, 0.1
    W, X = synth.make_quantizer_problem(21, m, n)
    ref = enc.spqr_quantize_from_calibration(W, X, bits, b1, b2, tau, lam)
    H = E.spqr_hessian(dev(X))
    U = E.spqr_inverse_cholesky(H, lam)
    got = E.spqr_quantize(dev(W), U, bits, b1, b2, tau)
    # another H^ic by rounding, so single decisions may differ: compare what the method is for
    err_ref = np.linalg.norm((W - ref.W_final) @ X)
    err_got = np.linalg.norm((W - got.W_final) @ X)
    assert abs(err_got - err_ref) <= 0.02 * err_ref
    assert abs(int(got.row_ptr[-1]) - int(ref.row_ptr[-1])) <= 0.02 * ref.row_ptr[-1] + 4
    assert (got.Q != ref.Q).mean() < 0.01
    # the encoder's output is a valid SpQR matrix: pack it, check it, multiply with it
    A = P.SpQRMatrix.from_logical(got)
    assert P.spqr_pack_check(A) == 0
    x = synth.make_x(n, 1, seed=(77,))
    y = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    want = orc.matvec(got, x)[0]
    assert np.linalg.norm(y - want) <= 1e-3 * np.linalg.norm(want)
    # and the decoder sees the weights the sweep left (outlier values are binary16)
    full = orc.reconstruct(got)
    assert np.abs(full - got.W_final).max() <= 2.0 ** -11 * np.abs(got.val.astype(np.float64)).max() + 1e-12
    torch.cuda.synchronize()


def test_act_order_and_permutations(E):
    import torch
    import paper_2306_03078_amd as P
    rng = np.random.default_rng(3)
    for n in (1, 5, 64, 200, 777, 2048):
        d = np.round(rng.uniform(0.5, 3.0, n), 2)          # rounding makes ties
        H = np.diag(d) + 0.0
        perm = E.spqr_act_order(dev(H)).cpu().numpy()
        assert np.array_equal(perm, enc.act_order(H)), n
    m, n = 64, 96
    W, X = synth.make_quantizer_problem(31, m, n)
    X = X * np.linspace(0.5, 3.0, n)[::-1, None] * np.where(np.arange(n) % 2, 1.0, 0.3)[:, None]
    Hd = E.spqr_hessian(dev(X))
    perm_d = E.spqr_act_order(Hd)
    perm = perm_d.cpu().numpy()
    Hn = Hd.cpu().numpy()
    assert np.array_equal(perm, enc.act_order(Hn))
    assert np.array_equal(E.spqr_permute_columns(dev(W), perm_d).cpu().numpy(), W[:, perm])
    assert np.array_equal(E.spqr_permute_symmetric(Hd, perm_d).cpu().numpy(), Hn[np.ix_(perm, perm)])
    # the whole chain with the heuristic, into the product kernel with its permuted input
    U = E.spqr_inverse_cholesky(E.spqr_permute_symmetric(Hd, perm_d), 0.05)
    got = E.spqr_quantize(E.spqr_permute_columns(dev(W), perm_d), U, 4, 16, 16, float("inf"))
    got.perm = perm
    A = P.SpQRMatrix.from_logical(got)
    assert P.spqr_pack_check(A) == 0
    x = (X[:, :1].T / np.abs(X).max()).astype(np.float16)     # a calibration input: what the error feedback protects
    y = P.spqr_gemv(A, dev(x[0])).cpu().numpy().astype(np.float64)
    want = orc.matvec(got, x)[0]
    assert np.linalg.norm(y - want) <= 1e-3 * np.linalg.norm(want)
    exact = W @ x[0].astype(np.float64)
    assert np.linalg.norm(y - exact) <= 0.1 * np.linalg.norm(exact)      # 4-bit weights: a few per cent
    torch.cuda.synchronize()


def test_argument_checks(E):
    import torch
    W = torch.zeros((64, 64), dtype=torch.float64, device="cuda:0")
    U = torch.eye(64, dtype=torch.float64, device="cuda:0")
    for kw in (dict(w_bits=1), dict(beta1=12), dict(beta2=48), dict(beta2=128), dict(w_bits=9)):
        args = dict(w_bits=3, beta1=16, beta2=16, tau=0.1)
        args.update(kw)
        with pytest.raises(Exception):
            E.spqr_quantize(W, U, **args)
    with pytest.raises(Exception):
        E.spqr_quantize(W[:60].contiguous(), U, 3, 16, 16, 0.1)        # m not a multiple of beta2
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(Exception):
        E.spqr_quantize(W, U, 3, 16, 16, 0.1, workspace=small)
    with pytest.raises(Exception):
        E.spqr_inverse_cholesky(U, 0.1, workspace=small)
