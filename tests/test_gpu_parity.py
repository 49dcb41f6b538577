"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle,
element by element on the same seeded inputs.

Bars: bit-exact codes, decoded statistics (binary32 reading) and CSR handling;
dense reconstruction within 1 binary16 ulp of the fp64 oracle; products within
relative L2 <= 1e-3 per output vector.
"""
import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_oracle as orc

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2306_03078_amd as P
    P.load_library()          # fails loudly if the HIP library is not built
    assert torch.cuda.is_available()
    return P


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def f16_ulp(v):
    """Spacing of binary16 at |v| (floor: the smallest normal's spacing)."""
    a = np.maximum(np.abs(v), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


# (w_bits, beta1, beta2, axis, tile-rows, tile-cols): several tiles, a ragged
# last block (tile columns not a multiple of 64) and more than one step per wave.
SHAPES = [
    (3, 16, 16, 1, 3, 70), (3, 16, 16, 0, 2, 130), (4, 16, 16, 1, 2, 200), (4, 16, 16, 0, 3, 65),
    (3, 8, 32, 1, 5, 67), (3, 8, 32, 0, 2, 1100), (4, 8, 32, 1, 2, 64), (4, 8, 32, 0, 1, 129),
    (3, 16, 16, 1, 1, 1), (3, 16, 16, 1, 2, 1100),
    (3, 16, 32, 0, 2, 5), (4, 32, 16, 1, 2, 9),          # no tuned kernel: generic path
    (3, 8, 64, 1, 5, 67), (3, 8, 64, 1, 3, 700), (3, 8, 64, 1, 1, 1),   # beta2 = 64: tiles of 8 x 64, column halves
    (3, 8, 64, 0, 1, 9), (4, 8, 64, 1, 2, 5),            # beta2 = 64 without a tuned kernel
]


def make(w, b1, b2, axis, ntr, ntc, rate=0.02, structure="uniform", seed=None):
    tr, tc = synth.tile_shape(b1, b2, axis)
    return synth.make_matrix(ntr * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis,
                             outlier_rate=rate, outlier_structure=structure,
                             seed=seed or (31, w, b1, b2, axis, ntr, ntc))


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", SHAPES)
def test_decode_is_bit_exact_and_dense_within_one_ulp(P, w, b1, b2, axis, ntr, ntc):
    f = make(w, b1, b2, axis, ntr, min(ntc, 130))
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    codes = P.spqr_dequant_dense(A, P.SPQR_OUT_CODES_U8).cpu().numpy()
    assert np.array_equal(codes, f.Q)
    s32, z32 = orc.decode_stats_f32(f)
    s_gpu = P.spqr_dequant_dense(A, P.SPQR_OUT_SCALE_F32).cpu().numpy()
    z_gpu = P.spqr_dequant_dense(A, P.SPQR_OUT_ZERO_F32).cpu().numpy()
    assert np.array_equal(s_gpu.view(np.uint32), s32.view(np.uint32))
    assert np.array_equal(z_gpu.view(np.uint32), z32.view(np.uint32))
    dense = orc.decode_dense(f)
    full = orc.reconstruct(f)
    d32 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F32).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(d32 - dense) <= 2.0 ** -20 * np.abs(dense) + 1e-30)
    d16 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F16).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(d16 - dense) <= f16_ulp(dense))
    o16 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F16 | P.SPQR_OUT_WITH_OUTLIERS).cpu().numpy()
    assert np.all(np.abs(o16.astype(np.float64) - full) <= f16_ulp(full))
    o32 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F32 | P.SPQR_OUT_WITH_OUTLIERS).cpu().numpy()
    assert np.all(np.abs(o32.astype(np.float64) - full) <= 2.0 ** -20 * np.abs(full) + 1e-7)
    # positions without an outlier are untouched by the outlier pass
    mask = np.ones(full.shape, bool)
    mask[orc.outlier_rows(f), f.col_idx.astype(np.int64)] = False
    assert np.array_equal(o16[mask], P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F16).cpu().numpy()[mask])


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", SHAPES)
def test_gemv_matches_oracle(P, w, b1, b2, axis, ntr, ntc):
    import torch
    f = make(w, b1, b2, axis, ntr, ntc)
    A = P.SpQRMatrix.from_logical(f)
    x = synth.make_x(f.n, 1, seed=(41, ntc))
    ref = orc.matvec(f, x)[0]
    y = P.spqr_gemv(A, dev(x[0]))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert rel_l2(y, ref) <= REL_L2, rel_l2(y, ref)
    # run-to-run determinism: fixed summation order, no atomics
    y2 = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    assert np.array_equal(y.view(np.uint32), y2.view(np.uint32))
    # fp16 output = RNE of the fp32 output
    yh = P.spqr_gemv(A, dev(x[0]), y_dtype=P.SPQR_F16).cpu().numpy()
    assert np.array_equal(yh.view(np.uint16), y.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("w,b1,b2,axis", [(3, 16, 16, 1), (3, 16, 16, 0), (4, 16, 16, 1), (3, 8, 32, 1),
                                          (3, 8, 32, 0), (3, 8, 64, 1)])
@pytest.mark.parametrize("b", [1, 2, 3, 4, 8, 16])
def test_smallbatch_matches_oracle(P, w, b1, b2, axis, b):
    f = make(w, b1, b2, axis, 3, 70)
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, b, seed=(43, b))
    ref = orc.matvec(f, X)
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    assert Y.shape == (b, f.m)
    for k in range(b):
        assert rel_l2(Y[k], ref[k]) <= REL_L2, (k, rel_l2(Y[k], ref[k]))
    # binary16 output = RNE of the binary32 output, on whichever path the batch takes
    Yh = P.spqr_gemm_smallbatch(A, dev(X), y_dtype=P.SPQR_F16).cpu().numpy()
    assert np.array_equal(Yh.view(np.uint16), Y.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("structure,rate", [("none", 0.0), ("rows8cols4", 0.03), ("cols64", 0.08),
                                            ("zipf", 0.02), ("uniform", 0.3), ("uniform", 0.003),
                                            ("uniform", 0.95), ("zipf", 0.2)])
@pytest.mark.parametrize("w,b1,b2,axis", [(3, 16, 16, 0), (3, 16, 16, 1), (3, 8, 32, 1), (4, 8, 32, 0), (3, 8, 64, 1)])
def test_outlier_structures(P, structure, rate, w, b1, b2, axis):
    # full rows, full columns, Zipf row counts, nearly empty rows (chunks spanning
    # several rows, empty rows) and strips with more entries than one round holds
    tr, tc = synth.tile_shape(b1, b2, axis)
    f = make(w, b1, b2, axis, 128 // tr, 1152 // tc, rate=rate, structure=structure)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    x = synth.make_x(f.n, 1, seed=(47,))
    y = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    assert rel_l2(y, orc.matvec(f, x)[0]) <= REL_L2
    # the outlier part alone (dense part switched off through zero statistics)
    f.s_s[:] = 0
    y = P.spqr_gemv(P.SpQRMatrix.from_logical(f), dev(x[0])).cpu().numpy()
    ref = orc.matvec_sparse_only(f, x)[0]
    assert np.linalg.norm(y - ref) <= 1e-5 * max(np.linalg.norm(ref), 1e-3)


@pytest.mark.parametrize("axis", [0, 1])
def test_special_cases(P, axis):
    f = make(3, 16, 16, axis, 2, 66, rate=0.02)
    x = synth.make_x(f.n, 1, seed=(53,))
    # zero codes and zero zero-point: only the outlier SpMV is left
    g = make(3, 16, 16, axis, 2, 66, rate=0.02)
    g.Q[:] = 0; g.z_q[:] = 0; g.z_z[:] = 0
    y = P.spqr_gemv(P.SpQRMatrix.from_logical(g), dev(x[0])).cpu().numpy()
    ref = orc.matvec_sparse_only(g, x)[0]
    assert rel_l2(y, ref) <= REL_L2
    # one-hot x extracts one column of W_hat.  With column groups the kernel
    # rounds s_hat*x_j to binary16 once (relative 2^-11 of the dense part); the
    # position-dependent code offsets (up to 128 against q/8) cancel in binary32
    # and leave up to ~1e-5 of the column's scale.
    A = P.SpQRMatrix.from_logical(f)
    W = orc.reconstruct(f)
    D = orc.decode_dense(f)
    for j in (0, 17, f.n - 1):
        e = np.zeros(f.n, np.float16); e[j] = 1.0
        y = P.spqr_gemv(A, dev(e)).cpu().numpy()
        assert np.all(np.abs(y - W[:, j]) <= 2.0 ** -11 * np.abs(D[:, j]) + 2e-5 * np.max(np.abs(D[:, j])))
        assert rel_l2(y, W[:, j]) <= REL_L2
    # all-zero x
    y = P.spqr_gemv(A, dev(np.zeros(f.n, np.float16))).cpu().numpy()
    assert np.all(y == 0)
    # negative and zero decoded scales are legal
    h = make(4, 16, 16, axis, 2, 10, rate=0.0)
    h.s_s[0, 0] = 0.0; h.s_s[1, 1] = -0.04
    xx = synth.make_x(h.n, 1, seed=(59,))
    y = P.spqr_gemv(P.SpQRMatrix.from_logical(h), dev(xx[0])).cpu().numpy()
    assert rel_l2(y, orc.matvec(h, xx)[0]) <= REL_L2


def test_input_permutation(P):
    f = make(3, 16, 16, 1, 2, 70)
    rng = np.random.default_rng(3)
    f.perm = rng.permutation(f.n).astype(np.int32)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    x = synth.make_x(f.n, 2, seed=(61,))
    Y = P.spqr_gemm_smallbatch(A, dev(x)).cpu().numpy()
    ref = orc.matvec(f, x)
    assert rel_l2(Y[0], ref[0]) <= REL_L2 and rel_l2(Y[1], ref[1]) <= REL_L2


def test_pack_check_finds_planted_format_errors(P):
    import torch
    f = make(3, 16, 16, 1, 2, 4, rate=0.05)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0

    def with_arrays(**kw):
        g = make(3, 16, 16, 1, 2, 4, rate=0.05)
        for k, v in kw.items():
            setattr(g, k, v)
        return P.SpQRMatrix.from_logical(g)

    rp = f.row_ptr.copy(); rp[5] = rp[4] - 1 if rp[4] > 0 else rp[6] + 1
    assert P.spqr_pack_check(with_arrays(row_ptr=rp)) == -6          # not monotone
    rp = f.row_ptr.copy(); rp[-1] -= 1
    assert P.spqr_pack_check(with_arrays(row_ptr=rp)) == -6          # does not end at nnz
    r = int(np.argmax(np.diff(f.row_ptr) >= 2)); a = int(f.row_ptr[r])
    col = f.col_idx.copy(); col[a], col[a + 1] = col[a + 1], col[a]
    assert P.spqr_pack_check(with_arrays(col_idx=col)) == -6         # columns not increasing
    col = f.col_idx.copy(); col[a + 1] = col[a]
    assert P.spqr_pack_check(with_arrays(col_idx=col)) == -6         # duplicate position
    col = f.col_idx.copy(); col[-1] = f.n
    assert P.spqr_pack_check(with_arrays(col_idx=col)) == -6         # column out of range
    val = f.val.copy(); val[3] = np.float16(np.inf)
    assert P.spqr_pack_check(with_arrays(val=val)) == -7
    assert P.spqr_pack_check(with_arrays(val=val), P.SPQR_CHECK_CSR) == 0
    zs = f.z_s.copy(); zs[1, 2] = np.float16(np.nan)
    assert P.spqr_pack_check(with_arrays(z_s=zs)) == -7
    perm = np.arange(f.n, dtype=np.int32); perm[7] = f.n
    assert P.spqr_pack_check(with_arrays(perm=perm)) == -3
    # O(1) descriptor checks in every entry point
    x = dev(synth.make_x(f.n, 1)[0])
    A.desc.packed_bytes -= 4
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemv(A, x)
    assert ei.value.status == -4
    A.desc.packed_bytes += 4
    A.desc.packed += 4
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemv(A, x)
    assert ei.value.status == -5
    A.desc.packed -= 4
    lib = P.load_library()
    import ctypes as C
    y = torch.empty(f.m, dtype=torch.float32, device="cuda:0")
    assert lib.spqr_gemm_smallbatch(C.byref(A.desc), x.data_ptr(), 257, y.data_ptr(), 0, None) == -8
    assert lib.spqr_gemm_smallbatch(C.byref(A.desc), x.data_ptr(), 0, y.data_ptr(), 0, None) == -8
    assert lib.spqr_gemv(C.byref(A.desc), x.data_ptr(), y.data_ptr(), 5, None) == -10
    assert lib.spqr_dequant_dense(C.byref(A.desc), 9, y.data_ptr(), None) == -10
    assert lib.spqr_dequant_dense(C.byref(A.desc), P.SPQR_OUT_CODES_U8 | 0x100, y.data_ptr(), None) == -10
    assert lib.spqr_gemv(C.byref(A.desc), None, y.data_ptr(), 0, None) == -1


@pytest.mark.parametrize("w,b1,b2,ntr,ntc", [(3, 16, 16, 2, 70), (4, 16, 16, 3, 130), (3, 8, 32, 2, 200), (4, 8, 32, 1, 65)])
def test_power_of_two_scaling_is_bit_exact_where_groups_run_along_rows(P, w, b1, b2, ntr, ntc):
    # group_axis 0 multiplies the codes with x itself (binary16 products are exact in binary32, the sums are
    # binary32 in a fixed order), so y(4x) == 4 y(x) bit for bit: scaling by a power of two commutes with every
    # rounding on the way.  (group_axis 1 rounds s_hat*x to binary16 first, which is not scale-invariant where
    # that product is subnormal; there the same call twice must still give the same bits.)
    f = make(w, b1, b2, 0, ntr, ntc, rate=0.03, structure="rows8cols4")
    A = P.SpQRMatrix.from_logical(f)
    x1 = synth.make_x(f.n, 1, seed=(67, w, b1))[0]
    y1 = P.spqr_gemv(A, dev(x1)).cpu().numpy()
    y4 = P.spqr_gemv(A, dev((x1 * np.float16(4)))).cpu().numpy()
    assert np.array_equal(y4.view(np.uint32), (np.float32(4) * y1).view(np.uint32))
    X = synth.make_x(f.n, 4, seed=(68, w, b1))
    Y1 = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    Y2 = P.spqr_gemm_smallbatch(A, dev(X * np.float16(2))).cpu().numpy()      # scaling up: exact in binary16 too
    assert np.array_equal(Y2.view(np.uint32), (np.float32(2) * Y1).view(np.uint32))


@pytest.mark.parametrize("axis", [0, 1])
def test_repeated_calls_give_the_same_bits_and_additivity(P, axis):
    f = make(3, 16, 16, axis, 2, 70, rate=0.03, structure="rows8cols4")
    A = P.SpQRMatrix.from_logical(f)
    x1 = synth.make_x(f.n, 1, seed=(67,))[0]; x2 = synth.make_x(f.n, 1, seed=(71,))[0]
    ya = P.spqr_gemv(A, dev(x1)).cpu().numpy()
    yb = P.spqr_gemv(A, dev(x1)).cpu().numpy()
    assert np.array_equal(ya.view(np.uint32), yb.view(np.uint32))
    X = synth.make_x(f.n, 16, seed=(69,))
    Ya = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    Yb = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    assert np.array_equal(Ya.view(np.uint32), Yb.view(np.uint32))
    xs = (x1.astype(np.float32) + x2.astype(np.float32)).astype(np.float16)
    ys = P.spqr_gemv(A, dev(xs)).cpu().numpy()
    assert rel_l2(ys, orc.matvec(f, xs)[0]) <= REL_L2


def test_runs_on_a_side_stream(P):
    import torch
    f = make(3, 16, 16, 1, 2, 70)
    A = P.SpQRMatrix.from_logical(f)
    x = dev(synth.make_x(f.n, 1, seed=(73,))[0])
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        y = P.spqr_gemv(A, x, stream=s)
    s.synchronize()
    assert rel_l2(y.cpu().numpy(), orc.matvec(f, synth.make_x(f.n, 1, seed=(73,)))[0]) <= REL_L2


@pytest.mark.parametrize("w,b1,b2,axis,ntc", [(3, 16, 16, 1, 70), (4, 16, 16, 0, 130), (3, 8, 32, 1, 67), (3, 8, 64, 1, 67),
                                              (3, 32, 16, 1, 9)])          # the last has no tuned kernel
def test_fused_projections_share_one_input(P, w, b1, b2, axis, ntc):
    """q/k/v-like: several matrices of different heights fed by one x, one call.
    Every matrix must match the oracle and, bit for bit, its own spqr_gemv."""
    import torch
    tr, tc = synth.tile_shape(b1, b2, axis)
    heights = (3, 1, 5, 2)                        # tile rows per matrix
    structures = ("uniform", "rows8cols4", "none", "zipf")
    fs = [synth.make_matrix(h * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis, outlier_rate=0.03,
                            outlier_structure=st, seed=(57, w, b1, axis, k))
          for k, (h, st) in enumerate(zip(heights, structures))]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    xh = synth.make_x(fs[0].n, 1, seed=(58, ntc))
    x = dev(xh[0])
    ys = P.spqr_gemv_fused(As, x)
    torch.cuda.synchronize()
    for f, A, y in zip(fs, As, ys):
        y = y.cpu().numpy()
        assert y.shape == (f.m,)
        assert rel_l2(y, orc.matvec(f, xh)[0]) <= REL_L2
        alone = P.spqr_gemv(A, x).cpu().numpy()
        assert rel_l2(y, alone) <= 1e-6            # same arithmetic; the launch plan may split a long strip differently
    # a single matrix, fp16 output, and the descriptor checks
    y1 = P.spqr_gemv_fused(As[:1], x, y_dtype=P.SPQR_F16)[0].cpu().numpy()
    assert np.array_equal(y1.view(np.uint16), P.spqr_gemv(As[0], x, y_dtype=P.SPQR_F16).cpu().numpy().view(np.uint16))
    other = P.SpQRMatrix.from_logical(synth.make_matrix(tr, (ntc + 1) * tc, w_bits=w, beta1=b1, beta2=b2,
                                                        group_axis=axis, outlier_rate=0.0, seed=(59,)))
    with pytest.raises(P.SpQRError):
        P.spqr_gemv_fused([As[0], other], x)      # different n
    with pytest.raises(P.SpQRError):
        P.spqr_gemv_fused(As * 3, x)              # more than SPQR_MAX_FUSED


def test_fused_projections_with_a_shared_permutation(P):
    import torch
    fs = []
    perm = np.random.default_rng(5).permutation(70 * 16).astype(np.int32)
    for k in range(2):
        f = make(3, 16, 16, 1, 2 + k, 70, seed=(61, k))
        f.perm = perm
        fs.append(f)
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    # descriptors must name the same device permutation
    As[1].desc.perm = As[0].desc.perm
    xh = synth.make_x(fs[0].n, 1, seed=(62,))
    ys = P.spqr_gemv_fused(As, dev(xh[0]))
    torch.cuda.synchronize()
    for f, y in zip(fs, ys):
        assert rel_l2(y.cpu().numpy(), orc.matvec(f, xh)[0]) <= REL_L2


@pytest.mark.parametrize("w,b1,b2,axis,ntc", [(3, 16, 16, 1, 70), (4, 16, 16, 0, 130), (3, 8, 32, 1, 40), (4, 8, 32, 0, 300)])
@pytest.mark.parametrize("b,mode", [(16, "1"), (7, "1"), (37, "1"), (16, "0"), (3, None), (1, None)])
def test_fused_batch_projections(P, monkeypatch, w, b1, b2, axis, ntc, b, mode):
    """spqr_gemm_fused: matrices of different heights (with and without outliers, with long rows) sharing a batch give
    what spqr_gemm_smallbatch gives one by one on the same path, and the oracle's result within the tolerance."""
    import torch
    if mode is not None:
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX if mode == "1" else P.SPQR_BATCH_PATH_VECTOR)
    tr, _ = synth.tile_shape(b1, b2, axis)
    specs = [(5, 0.03, "rows8cols4"), (2, 0.0, "none"), (9, 0.02, "zipf")]
    fs = [make(w, b1, b2, axis, ntr, ntc, rate=r, structure=st, seed=(96, i, ntc)) for i, (ntr, r, st) in enumerate(specs)]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    X = synth.make_x(fs[0].n, b, seed=(97, b))
    Ys = P.spqr_gemm_fused(As, dev(X))
    torch.cuda.synchronize()
    for f, A, Y in zip(fs, As, Ys):
        Y = Y.cpu().numpy()
        ref = orc.matvec(f, X)
        assert Y.shape == (b, f.m)
        assert max(rel_l2(Y[k], ref[k]) for k in range(b)) <= REL_L2
        # the same arithmetic; only the split of the steps (the order of the partial sums) may differ
        one = (P.spqr_gemm_smallbatch(A, dev(X)) if b > 1 else P.spqr_gemv(A, dev(X[0]))[None, :]).cpu().numpy()
        assert max(rel_l2(Y[k], one[k]) for k in range(b)) <= 1e-6
    Yh = P.spqr_gemm_fused(As, dev(X), y_dtype=P.SPQR_F16)
    for Y, H in zip(Ys, Yh):
        assert np.array_equal(H.cpu().numpy().view(np.uint16), Y.cpu().numpy().astype(np.float16).view(np.uint16))


def test_fused_batch_projections_with_a_shared_permutation_and_argument_checks(P, monkeypatch):
    import torch
    import ctypes as C
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    perm = np.random.default_rng(6).permutation(70 * 16).astype(np.int32)
    fs = []
    for i, ntr in enumerate((3, 6)):
        f = make(3, 16, 16, 1, ntr, 70, rate=0.02, seed=(98, i))
        f.perm = perm
        fs.append(f)
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    As[1].desc.perm = As[0].desc.perm          # descriptors must name the same device permutation
    X = synth.make_x(fs[0].n, 16, seed=(99,))
    Ys = P.spqr_gemm_fused(As, dev(X))
    torch.cuda.synchronize()
    for f, Y in zip(fs, Ys):
        ref = orc.matvec(f, X)
        assert max(rel_l2(Y.cpu().numpy()[k], ref[k]) for k in range(16)) <= REL_L2
    other = P.SpQRMatrix.from_logical(make(4, 16, 16, 1, 2, 70, seed=(98, 9)))
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemm_fused([As[0], other], dev(X))
    assert ei.value.status == -3
    lib = P.load_library()
    descs = (C.POINTER(type(As[0].desc)) * 1)(C.pointer(As[0].desc))
    ys = (C.c_void_p * 1)(Ys[0].data_ptr())
    assert lib.spqr_gemm_fused(descs, 1, dev(X).data_ptr(), 0, ys, 0, None) == -8
    assert lib.spqr_gemm_fused(descs, 9, dev(X).data_ptr(), 4, ys, 0, None) == -3


def test_fallback_kernel_agrees_with_the_tuned_one(P, monkeypatch):
    """The option SPQR_OPT_FORCE_GENERIC sends a tuned shape through the element-wise fallback kernel."""
    f = make(3, 16, 16, 1, 2, 70, rate=0.03, structure="rows8cols4")
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, 3, seed=(67,))
    ref = orc.matvec(f, X)
    tuned = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    P.spqr_set_option(P.SPQR_OPT_FORCE_GENERIC, 1)
    slow = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    fused = [y.cpu().numpy() for y in P.spqr_gemv_fused([A, A], dev(X[0]))]
    P.spqr_set_option(P.SPQR_OPT_FORCE_GENERIC, 0)
    for k in range(3):
        assert rel_l2(slow[k], ref[k]) <= 1e-5          # canonical binary32 decode, x used exactly
        assert rel_l2(tuned[k], slow[k]) <= REL_L2
    assert all(rel_l2(y, ref[0]) <= 1e-5 for y in fused)


def test_seeded_random_geometries_and_outlier_mixes(P):
    """Many small seeded cases: every tuned tile shape and width, ragged blocks, one to many steps
    per wavefront, batches 1-5, all outlier structures at rates from none to dense rows."""
    import torch
    rng = np.random.default_rng(20240607)
    shapes = [(16, 16, 1), (16, 16, 0), (8, 32, 1), (8, 32, 0)]
    structures = ["none", "uniform", "rows8cols4", "cols64", "zipf"]
    worst = 0.0
    for case in range(48):
        b1, b2, axis = shapes[case % 4]
        w = 3 + (case // 4) % 2
        ntr = int(rng.integers(1, 5))
        ntc = int(rng.choice([1, 3, 63, 64, 65, 127, 129, 200, 257, 515, 1030]))
        st = structures[case % 5]
        rate = 0.0 if st == "none" else float(rng.choice([0.002, 0.01, 0.05, 0.3]))
        f = make(w, b1, b2, axis, ntr, ntc, rate=rate, structure=st, seed=(71, case))
        A = P.SpQRMatrix.from_logical(f)
        assert P.spqr_pack_check(A) == 0
        b = int(rng.integers(1, 6))
        X = synth.make_x(f.n, b, seed=(72, case))
        ref = orc.matvec(f, X)
        Y = (P.spqr_gemv(A, dev(X[0]))[None, :] if b == 1 else P.spqr_gemm_smallbatch(A, dev(X))).cpu().numpy()
        torch.cuda.synchronize()
        for k in range(b):
            err = rel_l2(Y[k], ref[k])
            worst = max(worst, err)
            assert err <= REL_L2, (case, w, b1, b2, axis, ntr, ntc, st, rate, b, k, err)
    assert worst > 0.0


@pytest.mark.parametrize("w,axis,ntr,ntc", [(3, 1, 3, 70), (4, 1, 2, 200), (3, 0, 2, 130), (4, 0, 7, 65),
                                            (3, 1, 1, 1), (4, 1, 4, 1100)])
@pytest.mark.parametrize("b", [5, 8, 13, 16])
def test_matrix_core_batch_path(P, monkeypatch, w, axis, ntr, ntc, b):
    """Batches above 4 on 16x16 tiles: dense part on the matrix cores (weights dequantised
    to binary16, one rounding; several strips per workgroup, ragged last workgroup), outliers
    added by a pass of their own.  Checked against the oracle and against the vector path
    (SPQR_OPT_BATCH_PATH) on the same inputs.  The shapes cover one and many steps, steps split over
    workgroups with partial results, strips whose outliers pass through LDS in several chunks."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(w, 16, 16, axis, ntr, ntc, rate=0.03, structure="rows8cols4" if ntc > 64 else "uniform")
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, b, seed=(47, b, ntc))
    ref = orc.matvec(f, X)
    Y = P.spqr_gemm_smallbatch(A, dev(X))
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    assert Y.shape == (b, f.m) and np.all(np.isfinite(Y))
    for k in range(b):
        assert rel_l2(Y[k], ref[k]) <= REL_L2, (k, rel_l2(Y[k], ref[k]))
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_VECTOR)
    Yv = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    for k in range(b):
        assert rel_l2(Y[k], Yv[k]) <= REL_L2
    # deterministic
    Y2 = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    assert np.array_equal(Y.view(np.uint32), Y2.view(np.uint32))


@pytest.mark.parametrize("w,axis,ntr,ntc", [(3, 1, 5, 70), (4, 1, 17, 33), (3, 0, 3, 130), (4, 0, 9, 300), (3, 1, 1, 9),
                                            (3, 0, 1, 20), (4, 1, 8, 140)])
@pytest.mark.parametrize("b", [5, 16, 23])
def test_matrix_core_batch_path_8x32_tiles(P, monkeypatch, w, axis, ntr, ntc, b):
    """beta1 = 8, beta2 = 32: tiles of 8 rows x 32 columns (groups along the rows, 8 strips per workgroup, an odd
    number of strips leaves m % 16 == 8) and of 32 x 8 (groups along the columns, two blocks of 16 rows per tile)."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(w, 8, 32, axis, ntr, ntc, rate=0.03, structure="rows8cols4" if ntc > 64 else "uniform", seed=(89, ntr, ntc))
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, b, seed=(90, b, ntc))
    ref = orc.matvec(f, X)
    Y = P.spqr_gemm_smallbatch(A, dev(X))
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    assert Y.shape == (b, f.m) and np.all(np.isfinite(Y))
    for k in range(b):
        assert rel_l2(Y[k], ref[k]) <= REL_L2, (k, rel_l2(Y[k], ref[k]))
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_VECTOR)
    Yv = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    for k in range(b):
        assert rel_l2(Y[k], Yv[k]) <= REL_L2


@pytest.mark.parametrize("structure,rate", [("zipf", 0.05), ("cols64", 0.08), ("rows8cols4", 0.3), ("uniform", 0.95),
                                            ("uniform", 0.2), ("zipf", 0.3)])
def test_matrix_core_batch_path_outlier_mixes(P, monkeypatch, structure, rate):
    """The finishing kernel of the batch path: rows dealt to all lanes, rows cut into parts that
    cross a chunk of staged entries (rate 0.2: 16 rows of about 416), nearly dense CSR."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(4, 16, 16, 1, 5, 130, rate=rate, structure=structure, seed=(81, int(rate * 100)))
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, 11, seed=(82,))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    ref = orc.matvec(f, X)
    assert max(rel_l2(Y[k], ref[k]) for k in range(11)) <= REL_L2


@pytest.mark.parametrize("ntc,rate", [(138, 0.95), (300, 0.45), (600, 0.45), (40, 0.9)])
def test_matrix_core_long_rows_back_to_back(P, monkeypatch, ntc, rate):
    """Every row about as long as the next (2098, 2160, 4320, 576 entries): none of them is far above the average,
    so all stay in the finishing kernel, in 16 parts of up to 270 entries that cross the chunks of staged entries."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(3, 16, 16, 0, 3, ntc, rate=rate, structure="uniform", seed=(83, ntc))
    assert np.diff(f.row_ptr).min() > 512
    A = P.SpQRMatrix.from_logical(f)
    for b in (16, 7):
        X = synth.make_x(f.n, b, seed=(84, b))
        Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        ref = orc.matvec(f, X)
        assert max(rel_l2(Y[k], ref[k]) for k in range(b)) <= REL_L2


def test_matrix_core_long_rows_many_rows_per_workgroup(P, monkeypatch):
    """A tall matrix whose rows 31, 32, 63, 64 and 79 of every 80 hold 700 outliers, the others none: a workgroup
    that takes long rows looks at 255 rows at a time and keeps which of them are long in one 64-bit mask per
    wavefront (row 31 of a wavefront's 64 is bit 31 of the mask's low word, rows 63 / 64 the seam between two
    wavefronts' masks)."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(3, 16, 16, 1, 640, 48, rate=0.0, structure="none", seed=(85,))
    assert f.m == 10240 and f.n == 768
    rng = np.random.default_rng(85)
    counts = np.zeros(f.m, np.int64)
    counts[np.isin(np.arange(f.m) % 80, (31, 32, 63, 64, 79))] = 700
    f.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    f.col_idx = np.concatenate([np.sort(rng.choice(f.n, size=c, replace=False)) for c in counts if c]).astype(np.uint16)
    f.val = rng.standard_normal(f.col_idx.shape[0]).astype(np.float16)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    X = synth.make_x(f.n, 9, seed=(86,))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    ref = orc.matvec(f, X)
    assert max(rel_l2(Y[k], ref[k]) for k in range(9)) <= REL_L2


def _with_row_counts(f, counts, seed):
    """Replaces the outliers of f by rows of the given lengths (sorted random columns, normal values)."""
    rng = np.random.default_rng(seed)
    f.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    f.col_idx = np.concatenate([np.sort(rng.choice(f.n, size=int(c), replace=False)) for c in counts if c]).astype(np.uint16)
    f.val = rng.standard_normal(f.col_idx.shape[0]).astype(np.float16)
    return f


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", [(3, 16, 16, 1, 40, 140), (4, 8, 32, 1, 80, 70)])
def test_matrix_core_long_rows_shared_out_by_entries(P, monkeypatch, w, b1, b2, axis, ntr, ntc):
    """The long-row workgroups own equal shares of the entry indices, whatever the rows: a block of heavy rows next
    to each other (full rows, rows of 513, 1024 and 1025 entries: one entry into a new slice, exact slices), rows
    just at and just above what counts as long (256 / 257 entries), empty rows between them, and shares whose
    bounds fall inside a row, on a slice bound and on a row bound."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(w, b1, b2, axis, ntr, ntc, rate=0.0, structure="none", seed=(120, w))
    assert f.n == 2240
    counts = np.zeros(f.m, np.int64)
    counts[100:108] = f.n                      # eight full rows in a block
    counts[108] = 513
    counts[110] = 1024
    counts[111] = 1025
    counts[300] = 256                          # not long: stays with the finishing kernel
    counts[301] = 257                          # long
    counts[f.m - 1] = 2000                     # the last row
    counts[::7] += 3                           # a few entries in every 7th row
    counts = np.minimum(counts, f.n)
    _with_row_counts(f, counts, 120)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    for b in (5, 16):
        X = synth.make_x(f.n, b, seed=(121, b))
        Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        ref = orc.matvec(f, X)
        assert max(rel_l2(Y[k], ref[k]) for k in range(b)) <= REL_L2, (w, b)


def test_matrix_core_long_rows_of_a_very_tall_matrix(P, monkeypatch):
    """More than 65536 rows: the search for a share's first row takes two rounds of probes.  Long rows at the very
    top, around the probes' first bracket and at the bottom; the oracle is sampled on those rows and 64 others."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(3, 16, 16, 1, 4200, 20, rate=0.0, structure="none", seed=(122,))
    assert f.m == 67200 and f.n == 320
    counts = np.zeros(f.m, np.int64)
    heavy = (0, 1, 255, 256, 257, 262, 263, 30000, 65535, 65536, 67198, 67199)
    counts[list(heavy)] = 300
    counts[1000:60000:97] = 2
    _with_row_counts(f, counts, 122)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    X = synth.make_x(f.n, 7, seed=(123,))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    rows = np.unique(np.concatenate([np.array(heavy), np.arange(1000, 60000, 97)[:32], np.random.default_rng(5).integers(0, f.m, 32)]))
    ref = orc.matvec_rows(f, X, rows)
    assert max(rel_l2(Y[k][rows], ref[k]) for k in range(7)) <= REL_L2


def test_batch_scratch_is_kept_per_stream_grows_and_falls_back(P, monkeypatch):
    """The batch path keeps one scratch buffer per stream: a small call, then a larger one on the same stream (the
    buffer grows), calls on two streams in turn, and more streams than the library keeps buffers for (the rest
    allocate stream-ordered).  Every result against the oracle."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    small = make(3, 16, 16, 1, 4, 70, rate=0.02, structure="uniform", seed=(130,))
    large = make(4, 16, 16, 1, 24, 140, rate=0.02, structure="uniform", seed=(131,))
    As = {id(f): P.SpQRMatrix.from_logical(f) for f in (small, large)}
    Xs = {id(f): synth.make_x(f.n, 16, seed=(132, f.n)) for f in (small, large)}
    refs = {id(f): orc.matvec(f, Xs[id(f)]) for f in (small, large)}
    streams = [torch.cuda.Stream() for _ in range(11)]
    torch.cuda.synchronize()
    outs = []
    for f in (small, large, small):            # the same stream: grows once, then reused
        with torch.cuda.stream(streams[0]):
            outs.append((f, P.spqr_gemm_smallbatch(As[id(f)], dev(Xs[id(f)]))))
    for k in range(6):                         # two streams in turn
        f = (small, large)[k % 2]
        with torch.cuda.stream(streams[1 + k % 2]):
            outs.append((f, P.spqr_gemm_smallbatch(As[id(f)], dev(Xs[id(f)]))))
    for st in streams[3:]:                     # 8 more streams: beyond the kept buffers
        with torch.cuda.stream(st):
            outs.append((large, P.spqr_gemm_smallbatch(As[id(large)], dev(Xs[id(large)]))))
    torch.cuda.synchronize()
    for f, Y in outs:
        Y = Y.cpu().numpy()
        assert max(rel_l2(Y[k], refs[id(f)][k]) for k in range(16)) <= REL_L2


def test_batch_calls_from_two_host_threads_on_one_stream(P, monkeypatch):
    """Two host threads enqueue batch calls on the same stream at the same time: the calls share the stream's scratch
    buffer, whose lock keeps their kernels from interleaving.  Every result against the oracle."""
    import threading
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    fs = [make(3, 16, 16, 1, 6, 70, rate=0.02, structure="uniform", seed=(140,)),
          make(4, 16, 16, 1, 10, 140, rate=0.02, structure="uniform", seed=(141,))]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    Xs = [dev(synth.make_x(f.n, 16, seed=(142, f.n))) for f in fs]
    refs = [orc.matvec(f, X.cpu().numpy()) for f, X in zip(fs, Xs)]
    stream = torch.cuda.current_stream()
    outs = [[], []]
    errors = []

    def work(k):
        try:
            for _ in range(25):
                outs[k].append(P.spqr_gemm_smallbatch(As[k], Xs[k], stream=stream))
        except Exception as e:                 # a failure in a thread must fail the test
            errors.append(e)

    threads = [threading.Thread(target=work, args=(k,)) for k in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for k in (0, 1):
        first = outs[k][0]
        assert max(rel_l2(first.cpu().numpy()[j], refs[k][j]) for j in range(16)) <= REL_L2
        for Y in outs[k][1:]:
            assert torch.equal(Y, first)       # deterministic: every call gives the same bits


def test_batch_path_in_a_captured_graph_replays_like_the_eager_call(P, monkeypatch):
    """Captured, the batch path allocates its scratch stream-ordered (allocation nodes of the graph).  Several
    replays with eager calls and synchronisations in between, each compared bit for bit with the eager result."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(4, 16, 16, 1, 12, 140, rate=0.02, structure="uniform", seed=(133,))
    A = P.SpQRMatrix.from_logical(f)
    X = dev(synth.make_x(f.n, 16, seed=(134,)))
    eager = P.spqr_gemm_smallbatch(A, X).clone()
    ref = orc.matvec(f, X.cpu().numpy())
    assert max(rel_l2(eager.cpu().numpy()[k], ref[k]) for k in range(16)) <= REL_L2
    Y = torch.zeros_like(eager)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.spqr_gemm_smallbatch(A, X, out=Y)
    for rep in range(4):
        Y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager), rep
        other = P.spqr_gemm_smallbatch(A, X)       # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(other, eager), rep


def test_matrix_core_long_rows_next_to_rows_like_the_average(P, monkeypatch):
    """What counts as a long row depends on the average: with 30 % outliers everywhere (about 600 per row) plus two
    full rows of 2080, only the full rows leave the finishing kernel; the others are cut into 16 parts of about 39."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(4, 16, 16, 1, 5, 130, rate=0.3, structure="uniform", seed=(94,))
    rng = np.random.default_rng(94)
    counts = np.diff(f.row_ptr).astype(np.int64)
    rows = [np.sort(f.col_idx[f.row_ptr[r]:f.row_ptr[r + 1]]) for r in range(f.m)]
    vals = [f.val[f.row_ptr[r]:f.row_ptr[r + 1]] for r in range(f.m)]
    for r in (7, 40):
        rows[r] = np.arange(f.n, dtype=np.uint16)
        vals[r] = rng.standard_normal(f.n).astype(np.float16)
        counts[r] = f.n
    f.row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    f.col_idx = np.concatenate(rows).astype(np.uint16)
    f.val = np.concatenate(vals).astype(np.float16)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    X = synth.make_x(f.n, 12, seed=(95,))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    ref = orc.matvec(f, X)
    assert max(rel_l2(Y[k], ref[k]) for k in range(12)) <= REL_L2


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", [(3, 16, 16, 1, 3, 70), (4, 16, 16, 0, 2, 130), (3, 8, 32, 1, 5, 40),
                                                  (4, 8, 32, 0, 2, 300)])
@pytest.mark.parametrize("b", [6, 16])
def test_matrix_core_batch_path_with_permutation_and_f16_output(P, monkeypatch, w, b1, b2, axis, ntr, ntc, b):
    """Act-order input permutation (column j of the matrix meets x[perm[j]]) and binary16 output on the batch path,
    with and without outliers, one and several splits of the steps."""
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    for rate in (0.03, 0.0):
        f = make(w, b1, b2, axis, ntr, ntc, rate=rate, structure="uniform" if rate else "none", seed=(91, ntc, int(rate * 100)))
        f.perm = np.random.default_rng(92 + ntc).permutation(f.n).astype(np.int32)
        A = P.SpQRMatrix.from_logical(f)
        X = synth.make_x(f.n, b, seed=(93, b))
        ref = orc.matvec(f, X)
        Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        assert max(rel_l2(Y[k], ref[k]) for k in range(b)) <= REL_L2
        Yh = P.spqr_gemm_smallbatch(A, dev(X), y_dtype=P.SPQR_F16).cpu().numpy()
        assert np.array_equal(Yh.view(np.uint16), Y.astype(np.float16).view(np.uint16))
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_VECTOR)
        Yv = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
        assert max(rel_l2(Y[k], Yv[k]) for k in range(b)) <= REL_L2


@pytest.mark.parametrize("b,mode", [(40, "1"), (33, "1"), (21, None), (64, "0")])
def test_batches_above_16_go_in_slices(P, monkeypatch, b, mode):
    """Slices of 16 on the matrix-core path (40 = 16 + 16 + 8; 33 leaves one vector), whatever the library's rule
    picks for a layer this small (21 = 16 on the matrix cores + 5 on the vector path), slices of 4 on the vector path."""
    if mode is not None:
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX if mode == "1" else P.SPQR_BATCH_PATH_VECTOR)
    f = make(4, 16, 16, 1, 3, 70, rate=0.03, structure="rows8cols4", seed=(87,))
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, b, seed=(88, b))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    ref = orc.matvec(f, X)
    assert Y.shape == (b, f.m)
    assert max(rel_l2(Y[k], ref[k]) for k in range(b)) <= REL_L2


def test_matrix_core_batch_path_without_outliers_and_sparse_only(P, monkeypatch):
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(3, 16, 16, 1, 2, 70, rate=0.0, structure="none")
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, 16, seed=(48,))
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    ref = orc.matvec(f, X)
    assert max(rel_l2(Y[k], ref[k]) for k in range(16)) <= REL_L2
    # codes and zero codes all 0 with z_z = 0: only the outliers are left
    g = make(4, 16, 16, 0, 2, 70, rate=0.05)
    g.Q[:] = 0; g.z_q[:] = 0; g.z_z[:] = 0
    B = P.SpQRMatrix.from_logical(g)
    Xg = synth.make_x(g.n, 8, seed=(49,))
    Yg = P.spqr_gemm_smallbatch(B, dev(Xg)).cpu().numpy()
    refg = orc.matvec_sparse_only(g, Xg)
    assert max(rel_l2(Yg[k], refg[k]) for k in range(8)) <= REL_L2
