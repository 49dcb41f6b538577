"""GPU parity of the two statistic variants of the ablations (Sec. 5): integer zero-point
(`SPQR_LAYOUT_ROUND_ZERO`) and 16-bit first-level statistics (`SPQR_LAYOUT_STATS16`), against the CPU oracle.

Same bars as the bilevel format: bit-exact codes and decoded statistics, dense reconstruction within one
binary16 ulp, products within relative L2 <= 1e-3 per output vector.
"""
import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_oracle as orc

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
LAYOUTS = ["round_zero", "stats16"]


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
    a = np.maximum(np.abs(v), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


def make(layout, w, b1, b2, axis, ntr, ntc, rate=0.02, structure="uniform"):
    tr, tc = synth.tile_shape(b1, b2, axis)
    return synth.make_matrix(ntr * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis, outlier_rate=rate,
                             outlier_structure=structure, seed=(61, w, b1, b2, axis, ntr, ntc), stat_layout=layout)


# tuned tiles of either orientation with ragged last blocks and several steps per wavefront, strips behind the
# last one of a two-strip workgroup (odd strip counts), and shapes without a tuned kernel (groups of 48: the
# ablation's own group size for 16-bit statistics)
SHAPES = [
    (3, 16, 16, 1, 3, 70), (3, 16, 16, 0, 2, 130), (4, 16, 16, 1, 2, 200), (4, 16, 16, 0, 3, 65),
    (3, 8, 32, 1, 5, 67), (3, 8, 32, 1, 3, 700), (3, 32, 8, 0, 2, 1100), (4, 8, 32, 1, 2, 64), (4, 32, 8, 0, 1, 129),
    (3, 16, 16, 1, 1, 1),
    (3, 48, 16, 0, 2, 9), (3, 48, 16, 1, 3, 5), (4, 8, 64, 1, 2, 3),
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", SHAPES)
def test_decode_is_bit_exact_and_dense_within_one_ulp(P, layout, w, b1, b2, axis, ntr, ntc):
    if (b1, b2) == (32, 8):
        b1, b2 = 8, 32
    f = make(layout, w, b1, b2, axis, ntr, min(ntc, 130))
    A = P.SpQRMatrix.from_logical(f)
    assert A.layout_version == {"round_zero": 2, "stats16": 3}[layout]
    assert P.spqr_pack_check(A) == 0
    assert np.array_equal(P.spqr_dequant_dense(A, P.SPQR_OUT_CODES_U8).cpu().numpy(), f.Q)
    s32, z32 = orc.decode_stats_f32(f)
    s_gpu = P.spqr_dequant_dense(A, P.SPQR_OUT_SCALE_F32).cpu().numpy()
    z_gpu = P.spqr_dequant_dense(A, P.SPQR_OUT_ZERO_F32).cpu().numpy()
    assert np.array_equal(s_gpu.view(np.uint32), s32.view(np.uint32))
    assert np.array_equal(z_gpu.view(np.uint32), z32.view(np.uint32))
    dense, full = orc.decode_dense(f), orc.reconstruct(f)
    d32 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F32).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(d32 - dense) <= 2.0 ** -20 * np.abs(dense) + 1e-30)
    o16 = P.spqr_dequant_dense(A, P.SPQR_OUT_DENSE_F16 | P.SPQR_OUT_WITH_OUTLIERS).cpu().numpy()
    assert np.all(np.abs(o16.astype(np.float64) - full) <= f16_ulp(full))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", SHAPES)
def test_gemv_matches_oracle(P, layout, w, b1, b2, axis, ntr, ntc):
    import torch
    if (b1, b2) == (32, 8):
        b1, b2 = 8, 32
    f = make(layout, w, b1, b2, axis, ntr, ntc)
    A = P.SpQRMatrix.from_logical(f)
    x = synth.make_x(f.n, 1, seed=(63, ntc))
    ref = orc.matvec(f, x)[0]
    y = P.spqr_gemv(A, dev(x[0]))
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert rel_l2(y, ref) <= REL_L2, rel_l2(y, ref)
    assert np.max(np.abs(y - ref)) <= 8e-3 * np.sqrt(np.mean(ref ** 2)) + 1e-6
    y2 = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    assert np.array_equal(y.view(np.uint32), y2.view(np.uint32))
    yh = P.spqr_gemv(A, dev(x[0]), y_dtype=P.SPQR_F16).cpu().numpy()
    assert np.array_equal(yh.view(np.uint16), y.astype(np.float16).view(np.uint16))
    # the fallback kernel on the same matrix
    P.spqr_set_option(P.SPQR_OPT_FORCE_GENERIC, 1)
    try:
        yg = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    finally:
        P.spqr_set_option(P.SPQR_OPT_FORCE_GENERIC, 0)
    assert rel_l2(yg, ref) <= REL_L2


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("w,b1,b2,axis", [(3, 16, 16, 1), (3, 16, 16, 0), (3, 8, 32, 1), (4, 8, 32, 0), (3, 48, 16, 0)])
@pytest.mark.parametrize("b", [2, 5, 16, 70])
def test_batches(P, layout, w, b1, b2, axis, b):
    # these layouts have no slices of 16: a few vectors run as passes of the batch-1 kernel, a dozen and more
    # through the dense copy (tiles of 256 codes), whatever the batch on the fallback kernel (groups of 48)
    f = make(layout, w, b1, b2, axis, 3, 70)
    A = P.SpQRMatrix.from_logical(f)
    X = synth.make_x(f.n, b, seed=(65, b))
    ref = orc.matvec(f, X)
    dense = b >= 12 and b1 * b2 == 256
    assert (P.spqr_workspace_bytes([A], b) >= 2 * f.m * f.n) == dense
    Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
    for k in range(b):
        assert rel_l2(Y[k], ref[k]) <= REL_L2, (k, rel_l2(Y[k], ref[k]))
    if not dense:                            # every vector of the batch is the batch-1 result, bit for bit
        y0 = P.spqr_gemv(A, dev(X[b - 1])).cpu().numpy()
        assert np.array_equal(Y[b - 1].view(np.uint32), y0.view(np.uint32))


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("axis,b1,b2", [(1, 8, 32), (0, 16, 16)])
def test_grouped_and_fused_calls(P, layout, axis, b1, b2):
    # three projections of one format in one launch, own inputs (grouped) and a shared input (fused)
    tr, tc = synth.tile_shape(b1, b2, axis)
    n = 40 * tc
    fs = [synth.make_matrix(k * tr, n, w_bits=3, beta1=b1, beta2=b2, group_axis=axis, outlier_rate=0.02,
                            seed=(67, k, axis), stat_layout=layout) for k in (5, 3, 8)]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    xs = [synth.make_x(n, 1, seed=(69, i))[0] for i in range(3)]
    ys = P.spqr_gemv_grouped(As, [dev(x) for x in xs])
    for f, A, x, y in zip(fs, As, xs, ys):
        y = y.cpu().numpy()
        assert rel_l2(y, orc.matvec(f, x)[0]) <= REL_L2
        assert np.array_equal(y.view(np.uint32), P.spqr_gemv(A, dev(x)).cpu().numpy().view(np.uint32))
    ys = P.spqr_gemv_fused(As, dev(xs[0]))
    for f, y in zip(fs, ys):
        assert rel_l2(y.cpu().numpy(), orc.matvec(f, xs[0])[0]) <= REL_L2
    # layouts do not mix in one call
    other = P.SpQRMatrix.from_logical(synth.make_matrix(2 * tr, n, w_bits=3, beta1=b1, beta2=b2, group_axis=axis,
                                                        outlier_rate=0.0, seed=(71,)))
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemv_fused([As[0], other], dev(xs[0]))
    assert ei.value.status == -3
    # the grouped call sorts them into launches by format
    fo = synth.make_matrix(2 * tr, n, w_bits=3, beta1=b1, beta2=b2, group_axis=axis, outlier_rate=0.0, seed=(71,))
    ym = P.spqr_gemv_grouped([As[0], other, As[1]], [dev(xs[0]), dev(xs[1]), dev(xs[2])])
    for f, x, y in zip((fs[0], fo, fs[1]), xs, ym):
        assert rel_l2(y.cpu().numpy(), orc.matvec(f, x)[0]) <= REL_L2


@pytest.mark.parametrize("layout", LAYOUTS)
def test_permutation_and_validation(P, layout):
    f = make(layout, 3, 16, 16, 1, 2, 70)
    rng = np.random.default_rng(5)
    f.perm = rng.permutation(f.n).astype(np.int32)
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A, P.SPQR_CHECK_CSR | P.SPQR_CHECK_NONFINITE | P.SPQR_CHECK_PERM) == 0
    x = synth.make_x(f.n, 1, seed=(73,))
    assert rel_l2(P.spqr_gemv(A, dev(x[0])).cpu().numpy(), orc.matvec(f, x)[0]) <= REL_L2
    # a non-finite 16-bit statistic is found wherever the layout keeps one
    g = make(layout, 3, 16, 16, 0, 2, 70)
    if layout == "stats16":
        g.z16[17, 3] = np.inf
    else:
        g.z_s[1, 69] = np.nan
    B = P.SpQRMatrix.from_logical(g)
    assert P.spqr_pack_check(B, P.SPQR_CHECK_NONFINITE) == -7


@pytest.mark.parametrize("layout", LAYOUTS)
def test_full_size_layer_whole_vector(P, layout):
    # a layer of the largest benchmark shape class (8192 x 8192, 3-bit, 8 x 32 tiles, 2 % outliers with 64 full columns)
    f = synth.make_matrix(8192, 8192, w_bits=3, beta1=8, beta2=32, group_axis=1, outlier_rate=0.02,
                          outlier_structure="cols64", seed=(75,), stat_layout=layout)
    A = P.SpQRMatrix.from_logical(f)
    x = synth.make_x(f.n, 1, seed=(77,))
    ref = orc.matvec(f, x)[0]
    y = P.spqr_gemv(A, dev(x[0])).cpu().numpy()
    assert rel_l2(y, ref) <= REL_L2, rel_l2(y, ref)
    assert np.max(np.abs(y - ref)) <= 8e-3 * np.sqrt(np.mean(ref ** 2))
