"""GPU tests of the entry points that take their scratch from the caller, of the grouped batch-1 call and of
spqr_pack_check on two streams.  Everything goes through the C ABI (ctypes binding)."""
import ctypes as C

import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

REL_L2 = 1e-3
GUARD = 4096


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


def make(w, b1, b2, axis, ntr, ntc, rate=0.02, structure="uniform", seed=None):
    tr, tc = synth.tile_shape(b1, b2, axis)
    return synth.make_matrix(ntr * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis,
                             outlier_rate=rate, outlier_structure=structure,
                             seed=seed or (41, w, b1, b2, axis, ntr, ntc))


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / np.linalg.norm(ref))


class Guarded:
    """A workspace of exactly `nbytes` with guard bytes in front and behind (the kernels must stay inside)."""

    def __init__(self, nbytes):
        import torch
        self.nbytes = int(nbytes)
        self.buf = torch.full((GUARD + self.nbytes + GUARD,), 0xA5, dtype=torch.uint8, device="cuda:0")
        assert self.buf.data_ptr() % 256 == 0
        self.ws = self.buf[GUARD:GUARD + self.nbytes] if self.nbytes else None

    def intact(self):
        import torch
        torch.cuda.synchronize()
        return bool((self.buf[:GUARD] == 0xA5).all()) and bool((self.buf[GUARD + self.nbytes:] == 0xA5).all())


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc,structure,rate", [
    (3, 16, 16, 1, 5, 140, "uniform", 0.02), (4, 16, 16, 0, 9, 300, "zipf", 0.05), (3, 8, 32, 1, 17, 67, "cols64", 0.08),
    (4, 8, 32, 0, 2, 700, "rows8cols4", 0.3), (3, 16, 16, 1, 2, 70, "none", 0.0)])
@pytest.mark.parametrize("b", [5, 16, 37])
def test_caller_workspace_gives_the_library_scratch_results(P, w, b1, b2, axis, ntr, ntc, structure, rate, b):
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(w, b1, b2, axis, ntr, ntc, rate=rate, structure=structure)
    A = P.SpQRMatrix.from_logical(f)
    X = dev(synth.make_x(f.n, b, seed=(43, b)))
    need = P.spqr_workspace_bytes(A, b)
    assert need > 0
    g = Guarded(need)
    Y = P.spqr_gemm_smallbatch_ws(A, X, g.ws)
    assert g.intact()
    ref = orc.matvec(f, X.cpu().numpy())
    assert max(rel_l2(Y.cpu().numpy()[k], ref[k]) for k in range(b)) <= REL_L2
    assert torch.equal(Y, P.spqr_gemm_smallbatch(A, X))            # the same kernels, the same bits
    Yh = P.spqr_gemm_smallbatch_ws(A, X, g.ws, y_dtype=P.SPQR_F16)
    assert g.intact()
    assert torch.equal(Yh, P.spqr_gemm_smallbatch(A, X, y_dtype=P.SPQR_F16))


def test_caller_workspace_argument_checks(P):
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(3, 16, 16, 1, 4, 70)
    A = P.SpQRMatrix.from_logical(f)
    X = dev(synth.make_x(f.n, 16, seed=(44,)))
    need = P.spqr_workspace_bytes(A, 16)
    buf = torch.zeros(need + 512, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemm_smallbatch_ws(A, X, buf[:need - 256])
    assert ei.value.status == P.SPQR_ERR_WORKSPACE
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemm_smallbatch_ws(A, X, buf[16:16 + need])
    assert ei.value.status == -5
    with pytest.raises(P.SpQRError) as ei:
        P.spqr_gemm_smallbatch_ws(A, X, None)
    assert ei.value.status == P.SPQR_ERR_WORKSPACE
    # no scratch is needed where the vector kernel runs: a NULL workspace is fine
    assert P.spqr_workspace_bytes(A, 2) == 0
    Y2 = P.spqr_gemm_smallbatch_ws(A, X[:2].contiguous(), None)
    assert torch.equal(Y2, P.spqr_gemm_smallbatch(A, X[:2].contiguous()))
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_VECTOR)
    assert P.spqr_workspace_bytes(A, 16) == 0
    assert torch.equal(P.spqr_gemm_smallbatch_ws(A, X, None), P.spqr_gemm_smallbatch(A, X))


@pytest.mark.parametrize("w,b1,b2,axis,ntc", [(3, 16, 16, 1, 70), (4, 16, 16, 0, 130), (3, 8, 32, 1, 40), (4, 8, 32, 0, 300)])
@pytest.mark.parametrize("b", [7, 16, 21])
def test_fused_call_with_caller_workspace(P, w, b1, b2, axis, ntc, b):
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    fs = [make(w, b1, b2, axis, ntr, ntc, rate=r, structure=st, seed=(45, w, axis, ntr))
          for ntr, r, st in ((3, 0.02, "uniform"), (5, 0.2, "rows8cols4"), (2, 0.0, "none"))]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    X = dev(synth.make_x(fs[0].n, b, seed=(46, b)))
    need = P.spqr_workspace_bytes(As, b)
    assert need >= max(P.spqr_workspace_bytes(A, b) for A in As)
    g = Guarded(need)
    Ys = P.spqr_gemm_fused_ws(As, X, g.ws)
    assert g.intact()
    lib_Ys = P.spqr_gemm_fused(As, X)
    for f, Y, L in zip(fs, Ys, lib_Ys):
        ref = orc.matvec(f, X.cpu().numpy())
        assert max(rel_l2(Y.cpu().numpy()[k], ref[k]) for k in range(b)) <= REL_L2
        assert torch.equal(Y, L)


def _graph_node_types(capture):
    """Runs `capture(stream)` between hipStreamBeginCapture / EndCapture on a stream of its own and returns the
    node types of the captured graph, an executable instance and the graph (raw HIP handles)."""
    import torch
    hip = C.CDLL("libamdhip64.so")
    st = torch.cuda.Stream()
    sp = C.c_void_p(st.cuda_stream)
    with torch.cuda.stream(st):
        assert hip.hipStreamBeginCapture(sp, C.c_int(2)) == 0            # hipStreamCaptureModeRelaxed
        try:
            capture(st)
        finally:
            graph = C.c_void_p()
            rc = hip.hipStreamEndCapture(sp, C.byref(graph))
    assert rc == 0 and graph.value
    n = C.c_size_t(0)
    assert hip.hipGraphGetNodes(graph, None, C.byref(n)) == 0
    nodes = (C.c_void_p * n.value)()
    assert hip.hipGraphGetNodes(graph, nodes, C.byref(n)) == 0
    types = []
    for k in range(n.value):
        t = C.c_int(-1)
        assert hip.hipGraphNodeGetType(C.c_void_p(nodes[k]), C.byref(t)) == 0
        types.append(t.value)
    ex = C.c_void_p()
    assert hip.hipGraphInstantiate(C.byref(ex), graph, None, None, C.c_size_t(0)) == 0
    return types, ex, graph, st, hip


def test_captured_batch_call_with_caller_workspace_is_kernel_nodes_only(P):
    """Batch 16 through the workspace entry under stream capture: the graph holds kernel nodes and nothing else (no
    allocation, free or memset node), and every replay gives the eager result bit for bit."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    f = make(4, 16, 16, 1, 12, 140, rate=0.03, structure="rows8cols4", seed=(47,))
    A = P.SpQRMatrix.from_logical(f)
    X = dev(synth.make_x(f.n, 16, seed=(48,)))
    ws = torch.empty(P.spqr_workspace_bytes(A, 16), dtype=torch.uint8, device="cuda:0")
    eager = P.spqr_gemm_smallbatch_ws(A, X, ws).clone()
    ref = orc.matvec(f, X.cpu().numpy())
    assert max(rel_l2(eager.cpu().numpy()[k], ref[k]) for k in range(16)) <= REL_L2
    Y = torch.zeros_like(eager)
    torch.cuda.synchronize()
    types, ex, graph, st, hip = _graph_node_types(lambda s: P.spqr_gemm_smallbatch_ws(A, X, ws, out=Y, stream=s))
    assert len(types) >= 2 and all(t == 0 for t in types), types       # hipGraphNodeTypeKernel == 0
    for rep in range(4):
        Y.zero_()
        torch.cuda.synchronize()
        assert hip.hipGraphLaunch(ex, C.c_void_p(st.cuda_stream)) == 0
        torch.cuda.synchronize()
        assert torch.equal(Y, eager), rep
        P.spqr_gemm_smallbatch_ws(A, X, ws)                              # eager work between the replays
        torch.cuda.synchronize()
    assert hip.hipGraphExecDestroy(ex) == 0 and hip.hipGraphDestroy(graph) == 0


@pytest.mark.parametrize("w,b1,b2,axis", [(3, 8, 32, 1), (4, 16, 16, 1), (3, 8, 32, 0), (3, 8, 64, 1), (4, 16, 16, 0)])
def test_grouped_call_mixed_input_widths(P, w, b1, b2, axis):
    """Matrices of one format and different input widths in one grouped call: those of the width with the most
    strips size the launch; a narrower one rides along with the same plan, a wider one with the outlier products
    in the place of x (its workgroups' chunks fit one round by the hint on the longest row), and one whose hint
    understates its rows (set by hand here) still gives the right result, reading x from global memory."""
    import torch
    fs = [make(w, b1, b2, axis, 5, 200, rate=0.03, structure="cols64", seed=(80, 0)),
          make(w, b1, b2, axis, 9, 200, rate=0.02, structure="uniform", seed=(80, 1)),
          make(w, b1, b2, axis, 7, 400, rate=0.03, structure="uniform", seed=(80, 2)),      # wider: more chunks than threads
          make(w, b1, b2, axis, 4, 196, rate=0.02, structure="uniform", seed=(80, 3)),      # narrower
          make(w, b1, b2, axis, 6, 200, rate=0.0, structure="none", seed=(80, 4)),
          make(w, b1, b2, axis, 5, 400, rate=0.25, structure="rows8cols4", seed=(80, 5)),   # wider, hint understated below
          make(w, b1, b2, axis, 3, 40, rate=0.02, structure="uniform", seed=(80, 6))]       # too short for some plans
    if (w, b1, b2, axis) == (3, 8, 32, 1):
        # so wide that its x leaves less than a chunk per thread of the launch's LDS free (78336 bytes for this
        # plan: 12800 of x and a round of 2048 chunks), and far more chunks than a round: x from global memory
        fs.append(make(w, b1, b2, axis, 2, 1100, rate=0.25, structure="rows8cols4", seed=(80, 7)))
        fs.append(make(w, b1, b2, axis, 3, 300, rate=0.0, structure="none", seed=(80, 8)))   # wider, no outliers at all
        # wider, hint understated, between one and two rounds of the LDS behind its x (1648 chunks): rounds there
        fs.append(make(w, b1, b2, axis, 4, 400, rate=0.10, structure="uniform", seed=(80, 9)))
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    assert all(A.desc.max_row_nnz > 0 for A in As if A.desc.nnz > 0)
    for A in As[5:6] + As[7:8] + As[9:]:
        A.desc.max_row_nnz = 1
    xs = [dev(synth.make_x(f.n, 1, seed=(81, i))[0]) for i, f in enumerate(fs)]
    for y_dtype, tol in ((P.SPQR_F32, 1e-4), (P.SPQR_F16, 2e-3)):
        ys = P.spqr_gemv_grouped(As, xs, y_dtype=y_dtype)
        torch.cuda.synchronize()
        for i, (f, A, x, y) in enumerate(zip(fs, As, xs, ys)):
            one = P.spqr_gemv(A, x, y_dtype=y_dtype)
            if f.n == fs[0].n:
                assert torch.equal(y, one), i
            else:                                # another plan: the partial sums of a row meet in another order
                d = (y.double() - one.double()).abs().max().item()
                assert d <= tol * one.double().abs().max().item(), (i, d)
            assert rel_l2(y.cpu().numpy(), orc.matvec(f, x.cpu().numpy())[0]) <= REL_L2, i
    # few launches: the short matrix may have fewer steps than the plan has wavefronts per strip, a launch takes 8
    # matrices at most, the others share one
    outs = [torch.empty(f.m, dtype=torch.float32, device="cuda:0") for f in fs]
    types, ex, graph, st, hip = _graph_node_types(lambda s: P.spqr_gemv_grouped(As, xs, outs=outs, stream=s))
    assert 1 <= len(types) <= 3 and all(t == 0 for t in types), types    # hipGraphNodeTypeKernel == 0; 8 matrices per launch at most
    assert hip.hipGraphLaunch(ex, C.c_void_p(st.cuda_stream)) == 0
    torch.cuda.synchronize()
    for y, z in zip(P.spqr_gemv_grouped(As, xs), outs):
        assert torch.equal(y, z)
    assert hip.hipGraphExecDestroy(ex) == 0 and hip.hipGraphDestroy(graph) == 0
    # the same call twice gives the same bits
    again = P.spqr_gemv_grouped(As, xs)
    for y, z in zip(P.spqr_gemv_grouped(As, xs), again):
        assert torch.equal(y, z)


def test_grouped_call_equals_one_call_per_matrix(P):
    """All projections of a small decoder-block-like set, each with its own input: matrices of one format and width
    share a launch, a 4-bit one, one with a permutation and one without a tuned kernel take their own; every
    output equals spqr_gemv's bit for bit, and the oracle within tolerance."""
    import torch
    fs = [make(3, 8, 32, 1, 5, 70, rate=0.03, structure="cols64", seed=(50, 0)),
          make(3, 8, 32, 1, 9, 70, rate=0.02, structure="uniform", seed=(50, 1)),
          make(3, 8, 32, 1, 3, 200, rate=0.05, structure="rows8cols4", seed=(50, 2)),
          make(3, 8, 32, 1, 4, 70, rate=0.0, structure="none", seed=(50, 3)),
          make(4, 16, 16, 0, 3, 70, rate=0.02, structure="uniform", seed=(50, 4)),
          make(3, 8, 32, 1, 2, 70, rate=0.02, structure="uniform", seed=(50, 5)),
          make(3, 16, 32, 0, 2, 5, rate=0.02, structure="uniform", seed=(50, 6))]
    rng = np.random.default_rng(51)
    fs[5].perm = rng.permutation(fs[5].n).astype(np.int32)
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    xs = [dev(synth.make_x(f.n, 1, seed=(52, i))[0]) for i, f in enumerate(fs)]
    ys = P.spqr_gemv_grouped(As, xs)
    torch.cuda.synchronize()
    for f, A, x, y in zip(fs, As, xs, ys):
        assert torch.equal(y, P.spqr_gemv(A, x))
        assert rel_l2(y.cpu().numpy(), orc.matvec(f, x.cpu().numpy())[0]) <= REL_L2
    yh = P.spqr_gemv_grouped(As[:3], xs[:3], y_dtype=P.SPQR_F16)
    for A, x, y in zip(As, xs, yh):
        assert torch.equal(y, P.spqr_gemv(A, x, y_dtype=P.SPQR_F16))
    lib = P.load_library()
    k = 17
    descs = (C.POINTER(type(As[0].desc)) * k)(*[C.pointer(As[0].desc)] * k)
    ptrs = (C.c_void_p * k)(*[xs[0].data_ptr()] * k)
    outs = (C.c_void_p * k)(*[ys[0].data_ptr()] * k)
    assert lib.spqr_gemv_grouped(descs, 17, ptrs, outs, 0, None) == -3
    assert lib.spqr_gemv_grouped(descs, 0, ptrs, outs, 0, None) == -3
    assert lib.spqr_gemv_grouped(descs, 2, ptrs, None, 0, None) == -1


def test_pack_check_on_two_streams_at_once(P):
    """Every spqr_pack_check call has result words of its own: a valid and a broken matrix checked from two host
    threads on two streams keep their own verdicts."""
    import threading
    import torch
    good = make(3, 16, 16, 1, 40, 140, rate=0.05, seed=(53,))
    bad = make(3, 16, 16, 1, 40, 140, rate=0.05, seed=(54,))
    bad.col_idx = bad.col_idx.copy()
    a, b = int(bad.row_ptr[7]), int(bad.row_ptr[8])
    assert b - a >= 2
    bad.col_idx[a:b] = bad.col_idx[a:b][::-1]                       # columns of one row in falling order
    As = [P.SpQRMatrix.from_logical(good), P.SpQRMatrix.from_logical(bad)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [[], []]

    def work(k):
        for _ in range(30):
            got[k].append(P.spqr_pack_check(As[k], stream=streams[k]))

    threads = [threading.Thread(target=work, args=(k,)) for k in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert set(got[0]) == {0} and set(got[1]) == {-6}


def test_captured_fused_batch_call_takes_the_per_matrix_path(P):
    """spqr_gemm_fused on a capturing stream records one batch call per matrix (the fused launch set is kept out of
    graphs, see the skipped test below); replays must give what eager per-matrix calls give, bit for bit."""
    import torch
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    fs = [make(4, 16, 16, 1, ntr, 140, rate=0.03, structure=st, seed=(56, ntr)) for ntr, st in ((6, "uniform"), (9, "rows8cols4"))]
    As = [P.SpQRMatrix.from_logical(f) for f in fs]
    X = dev(synth.make_x(fs[0].n, 16, seed=(57,)))
    want = [P.spqr_gemm_smallbatch(A, X).clone() for A in As]
    ws = torch.empty(P.spqr_workspace_bytes(As, 16), dtype=torch.uint8, device="cuda:0")
    Ys = [torch.zeros_like(w) for w in want]
    torch.cuda.synchronize()
    types, ex, graph, st, hip = _graph_node_types(lambda s: P.spqr_gemm_fused_ws(As, X, ws, outs=Ys, stream=s))
    assert all(t == 0 for t in types), types
    for rep in range(3):
        for Y in Ys:
            Y.zero_()
        torch.cuda.synchronize()
        assert hip.hipGraphLaunch(ex, C.c_void_p(st.cuda_stream)) == 0
        torch.cuda.synchronize()
        for Y, w, f in zip(Ys, want, fs):
            assert torch.equal(Y, w), rep
    ref = [orc.matvec(f, X.cpu().numpy()) for f in fs]
    for Y, r in zip(Ys, ref):
        assert max(rel_l2(Y.cpu().numpy()[k], r[k]) for k in range(16)) <= REL_L2
    assert hip.hipGraphExecDestroy(ex) == 0 and hip.hipGraphDestroy(graph) == 0


@pytest.mark.skip(reason="GPU memory fault of unknown cause: a replay of a captured graph holding a whole decoder block "
                         "with six weight copies (42 calls, 12 of them spqr_gemm_fused on the fused matrix-core launch "
                         "set, scratch as allocation nodes) ended in a memory fault reported in the fused finishing "
                         "kernel.  Checked on the CPU since: the fused kernels use no private segment and 1248 bytes of "
                         "kernel arguments; every scratch offset of the launchers lies inside the exact-size workspace "
                         "(the guarded-workspace tests above run the same kernels eagerly on exact-size scratch). No "
                         "cause is shown, so the library keeps the fused launch set out of captured graphs and off "
                         "stream-ordered scratch, and this case stays off the GPU.")
def test_fused_launch_set_in_a_captured_decoder_block_graph(P):
    """The case that faulted, kept for the day a cause is known: it needs the library's guard in launch_gemm_fused
    (captured calls take the per-matrix path) lifted to mean anything."""
    import torch
    specs = synth.config_layers(2)
    mats = {sp.name: P.SpQRMatrix.from_logical(synth.make_config_layer(2, i, group_axis=1)) for i, sp in enumerate(specs)}
    copies = [{nm: (A if c == 0 else A.clone()) for nm, A in mats.items()} for c in range(6)]
    x_h = dev(synth.make_x(specs[0].n, 16, seed=(58,)))
    x_f = dev(synth.make_x(specs[-1].n, 16, seed=(59,)))
    outs = {nm: torch.empty((16, A.m), dtype=torch.float32, device="cuda:0") for nm, A in mats.items()}

    def block(c):
        P.spqr_gemm_fused([copies[c][nm] for nm in ("q", "k", "v")], x_h, outs=[outs[nm] for nm in ("q", "k", "v")])
        P.spqr_gemm_smallbatch(copies[c]["o"], x_h, out=outs["o"])
        P.spqr_gemm_fused([copies[c][nm] for nm in ("gate", "up")], x_h, outs=[outs[nm] for nm in ("gate", "up")])
        P.spqr_gemm_smallbatch(copies[c]["down"], x_f, out=outs["down"])

    block(0)
    torch.cuda.synchronize()
    eager = {nm: t.clone() for nm, t in outs.items()}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for c in range(6):
            block(c)
    for _ in range(3):
        g.replay()
        torch.cuda.synchronize()
        for nm in outs:
            assert torch.equal(outs[nm], eager[nm])
