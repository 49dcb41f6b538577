"""GPU parity at the full sizes of the five benchmark configurations, in the
launch configuration bench.py times.  Every output element of every distinct
layer and every batch a configuration names is compared with the oracle's full
fp64 decode + product (one layer at a time); codes and decoded statistics are
compared bit for bit over the whole matrix for one layer per configuration.
"""
import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

REL_L2 = 1e-3


@pytest.fixture(scope="module")
def P():
    import torch
    import paper_2306_03078_amd as P
    P.load_library()
    assert torch.cuda.is_available()
    return P


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def check_outputs(Y, ref, what):
    """Whole output vectors: relative L2 per vector, and every element against the scale of its vector."""
    Y = np.asarray(Y, dtype=np.float64)
    assert Y.shape == ref.shape, (what, Y.shape, ref.shape)
    assert np.all(np.isfinite(Y)), what
    worst = 0.0
    for k in range(ref.shape[0]):
        err = np.linalg.norm(Y[k] - ref[k]) / np.linalg.norm(ref[k])
        worst = max(worst, err)
        assert err <= REL_L2, (what, k, err)
        scale = np.sqrt(np.mean(ref[k] ** 2))
        bad = np.nonzero(np.abs(Y[k] - ref[k]) > 8 * REL_L2 * scale)[0]
        assert bad.size == 0, (what, k, bad[:8], Y[k][bad[:8]], ref[k][bad[:8]])
    return worst


def check_layer(P, f, batches, check_codes=False):
    import torch
    A = P.SpQRMatrix.from_logical(f)
    assert P.spqr_pack_check(A) == 0
    if check_codes:
        codes = P.spqr_dequant_dense(A, P.SPQR_OUT_CODES_U8).cpu().numpy()
        assert np.array_equal(codes, f.Q)
        del codes
        s32, z32 = orc.decode_stats_f32(f)
        assert np.array_equal(P.spqr_dequant_dense(A, P.SPQR_OUT_SCALE_F32).cpu().numpy().view(np.uint32),
                              s32.view(np.uint32))
        assert np.array_equal(P.spqr_dequant_dense(A, P.SPQR_OUT_ZERO_F32).cpu().numpy().view(np.uint32),
                              z32.view(np.uint32))
    # one oracle decode of the layer serves all its batches: the vectors of all batches as one stack
    Xs = [synth.make_x(f.n, b, seed=(77, b)) for b in batches]
    ref_all = orc.matvec(f, np.concatenate(Xs, axis=0))
    worst, at = 0.0, 0
    for b, X in zip(batches, Xs):
        ref = ref_all[at:at + b]
        at += b
        if b == 1:
            Y = P.spqr_gemv(A, dev(X[0])).cpu().numpy()[None, :]
        else:
            Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        torch.cuda.synchronize()
        worst = max(worst, check_outputs(Y, ref, (f.m, f.n, f.group_axis, b)))
    return worst


def distinct_layers(cfg):
    seen, out = set(), []
    for i, sp in enumerate(synth.config_layers(cfg)):
        if (sp.m, sp.n) not in seen:
            seen.add((sp.m, sp.n))
            out.append((i, sp))
    return out


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_llama7b_shaped_configs(P, cfg):
    for k, (i, sp) in enumerate(distinct_layers(cfg)):
        f = synth.make_config_layer(cfg, i, group_axis=1)
        check_layer(P, f, (1,), check_codes=(k == 0))
        del f
    # the paper's own orientation (groups along the input dimension) on the first layer
    f = synth.make_config_layer(cfg, 0, group_axis=0)
    check_layer(P, f, (1,))


def test_llama33b_shaped_config_with_batches(P):
    layers = distinct_layers(3)
    for k, (i, sp) in enumerate(layers):
        f = synth.make_config_layer(3, i, group_axis=1)
        check_layer(P, f, sp.batches, check_codes=(k == 0))
        del f
    f = synth.make_config_layer(3, 0, group_axis=0)
    check_layer(P, f, (1, 4))


def test_llama65b_shaped_config_resident_beside_filler(P):
    import torch
    # 60 GB of other allocations stay resident while the projections run (288 GB HBM sizing)
    filler = [torch.empty(6 * 1024 ** 3, dtype=torch.uint8, device="cuda:0") for _ in range(10)]
    for t in filler:
        t[:: 1 << 20].fill_(1)
    try:
        mats = []
        for k, (i, sp) in enumerate(distinct_layers(4)):
            f = synth.make_config_layer(4, i, group_axis=1)
            check_layer(P, f, sp.batches, check_codes=(k == 0))
            mats.append(P.SpQRMatrix.from_logical(f))      # keep the block's projections resident
            del f
        assert torch.cuda.memory_allocated() > 60 * 1024 ** 3
        f = synth.make_config_layer(4, 0, group_axis=0)
        check_layer(P, f, (1,))
    finally:
        del filler


def test_fused_projections_at_full_size(P):
    """q/k/v and gate/up of the LLaMA-7B-shaped block in one launch each, whole output vectors against the oracle."""
    import torch
    specs = synth.config_layers(2)
    for names in (("q", "k", "v"), ("gate", "up")):
        idx = [i for i, sp in enumerate(specs) if sp.name in names]
        fs = [synth.make_config_layer(2, i, group_axis=1) for i in idx]
        As = [P.SpQRMatrix.from_logical(f) for f in fs]
        X = synth.make_x(fs[0].n, 1, seed=(78, len(names)))
        X16 = synth.make_x(fs[0].n, 16, seed=(79, len(names)))
        ys = P.spqr_gemv_fused(As, dev(X[0]))
        # the same projections at batch 16 (the matrix-core path, one launch set for all of them)
        Ys = P.spqr_gemm_fused(As, dev(X16))
        torch.cuda.synchronize()
        for f, y, Y in zip(fs, ys, Ys):
            ref = orc.matvec(f, np.concatenate([X, X16], axis=0))
            check_outputs(y.cpu().numpy()[None, :], ref[:1], ("fused", f.m, f.n, 1))
            check_outputs(Y.cpu().numpy(), ref[1:], ("fused", f.m, f.n, 16))
        del fs, As


def test_large_batches_at_full_size(P):
    """256 and 64 vectors on the LLaMA-33B- and 65B-shaped layers (the dense-copy path, with and without split k):
    every output element against the oracle."""
    for cfg, name, b in ((3, "gate", 256), (3, "down", 256), (4, "q", 64), (4, "down", 128)):
        i = [k for k, sp in enumerate(synth.config_layers(cfg)) if sp.name == name][0]
        f = synth.make_config_layer(cfg, i, group_axis=1)
        A = P.SpQRMatrix.from_logical(f)
        assert P.spqr_workspace_bytes([A], b) >= 2 * f.m * f.n        # the path with the dense copy is the one taken
        X = synth.make_x(f.n, b, seed=(80, b))
        Y = P.spqr_gemm_smallbatch(A, dev(X)).cpu().numpy()
        check_outputs(Y, orc.matvec(f, X), ("dense copy", cfg, name, b))
        del f, A


@pytest.mark.parametrize("cfg", [4, 3, 2])
def test_grouped_block_at_full_size(P, cfg):
    """All seven projections of the LLaMA-65B-shaped block in one spqr_gemv_grouped call (what bench.py times: one
    launch, `down` with its products in the place of x), and of the LLaMA-33B- and 7B-shaped ones (one launch too:
    the workgroups of `down` that own rows of thousands of outliers go through rounds)."""
    import torch
    specs = synth.config_layers(cfg)
    fs = [synth.make_config_layer(cfg, i, group_axis=1) for i in range(len(specs))]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    xs = [synth.make_x(f.n, 1, seed=(81, i)) for i, f in enumerate(fs)]
    ys = P.spqr_gemv_grouped(As, [dev(x[0]) for x in xs])
    torch.cuda.synchronize()
    for f, x, y in zip(fs, xs, ys):
        check_outputs(y.cpu().numpy()[None, :], orc.matvec(f, x), ("grouped", f.m, f.n))


@pytest.mark.parametrize("layout", ["round_zero", "stats16"])
def test_statistic_variants_at_full_size(P, layout):
    """The two statistic layouts of the ablations on the largest layer shape and on a 7B-shaped one."""
    for cfg, i in ((4, 4), (1, 0)):
        f = synth.make_config_layer(cfg, i, group_axis=1, stat_layout=layout)
        check_layer(P, f, (1,), check_codes=True)
        del f
