"""Host-side logic of the library (no GPU): size model, packer round trip
through the oracle-side layout reader, descriptor validation, exported symbols."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2306_03078_amd as P
import spqr_synth as synth
from oracle import layout_reader, spqr_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(path):
    hdr = open(path).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return set(re.findall(r"\b(spqr_[a-z_0-9]+)\s*\(", hdr))


def test_library_exports_every_declared_symbol():
    names = _declared(os.path.join(ROOT, "include", "spqr.h"))
    assert {"spqr_pack_check", "spqr_gemv", "spqr_gemv_fused", "spqr_gemv_grouped", "spqr_gemm_fused", "spqr_gemm_smallbatch",
            "spqr_gemm_smallbatch_ws", "spqr_gemm_fused_ws", "spqr_workspace_bytes", "spqr_dequant_dense", "spqr_set_option",
            "spqr_pack_host", "spqr_packed_bytes", "spqr_pack_host_layout", "spqr_packed_bytes_layout", "spqr_strerror",
            "spqr_version"} <= names
    assert "spqr_plan_batch_steps" not in names      # a test hook, not part of the public interface
    enc = _declared(os.path.join(ROOT, "include", "spqr_encode.h"))
    assert {"spqr_hessian", "spqr_inverse_cholesky", "spqr_inverse_cholesky_workspace_bytes", "spqr_quantize",
            "spqr_quantize_workspace_bytes", "spqr_gather_outliers", "spqr_act_order", "spqr_act_order_workspace_bytes",
            "spqr_permute_columns", "spqr_permute_symmetric"} == enc
    names = names | enc
    hooks = _declared(os.path.join(ROOT, "paper_2306_03078_amd", "csrc", "spqr_test_hooks.h"))
    assert hooks == {"spqr_plan_batch_steps", "spqr_plan_grouped"}
    lib = C.CDLL(P.library_path())
    for nm in sorted(names | hooks):
        assert hasattr(lib, nm), nm


@pytest.mark.parametrize("w,b1,b2", [(3, 16, 16), (4, 16, 16), (3, 8, 32), (3, 16, 32), (3, 32, 16),
                                     (4, 8, 16), (3, 64, 64), (3, 128, 128), (3, 8, 16), (3, 32, 128)])
@pytest.mark.parametrize("axis", [0, 1])
def test_packed_size_is_the_papers_size_model(w, b1, b2, axis):
    # App. D Eq. 4 without outliers: b_w + (b_s+b_z)/beta1 + 64/(beta1*beta2), no padding.
    tr, tc = synth.tile_shape(b1, b2, axis)
    m, n = 3 * tr, 5 * tc
    nbytes = P.packed_bytes(m, n, w, 3, 3, b1, b2, axis)
    assert 8.0 * nbytes / (m * n) == orc.average_bits(w, 3, 3, b1, b2)


@pytest.mark.parametrize("w,b1,b2", [(3, 16, 16), (4, 16, 16), (3, 8, 32), (3, 48, 16), (4, 8, 64)])
@pytest.mark.parametrize("axis", [0, 1])
def test_packed_size_of_the_statistic_variants(w, b1, b2, axis):
    # Sec. 5 ablations: integer zero-point (one second-level pair per tile), 16-bit statistics (none); no padding.
    tr, tc = synth.tile_shape(b1, b2, axis)
    m, n = 3 * tr, 5 * tc
    assert 8.0 * P.packed_bytes(m, n, w, 3, 3, b1, b2, axis, P.SPQR_LAYOUT_ROUND_ZERO) / (m * n) \
        == orc.average_bits_round_zero(w, 3, 3, b1, b2)
    assert 8.0 * P.packed_bytes(m, n, w, 16, 16, b1, b2, axis, P.SPQR_LAYOUT_STATS16) / (m * n) \
        == orc.average_bits_stats16(w, b1)
    lib = P.load_library()
    assert lib.spqr_packed_bytes_layout(P.SPQR_LAYOUT_STATS16, m, n, w, 3, 3, b1, b2, axis) == -3
    assert lib.spqr_packed_bytes_layout(P.SPQR_LAYOUT_ROUND_ZERO, m, n, w, 16, 16, b1, b2, axis) == -3
    assert lib.spqr_packed_bytes_layout(4, m, n, w, 3, 3, b1, b2, axis) == -3
    assert lib.spqr_packed_bytes_layout(1, m, n, w, 3, 3, b1, b2, axis) == P.packed_bytes(m, n, w, 3, 3, b1, b2, axis)


def test_printed_bit_counts_for_config_tiles():
    # 3.625 bits (beta1=beta2=16) and 4 bits (beta1=8, beta2=32), App. C table.
    assert 8 * P.packed_bytes(4096, 4096, 3, 3, 3, 16, 16, 1) / 4096 ** 2 == 3.625
    assert 8 * P.packed_bytes(8192, 8192, 3, 3, 3, 8, 32, 1) / 8192 ** 2 == 4.0
    # an outlier costs 32 bits + the per-row 32-bit count: "32.03 to 32.1 bits" (Sec. 4.2)
    f = synth.make_matrix(4096, 4096, outlier_rate=0.01, seed=(0, 0))
    per_outlier = (f.col_idx.nbytes + f.val.nbytes + f.row_ptr.nbytes) * 8 / f.nnz
    assert 32.0 < per_outlier < 32.9


def test_unsupported_parameters_are_rejected():
    assert P.load_library().spqr_packed_bytes(64, 64, 5, 3, 3, 16, 16, 0) == -3
    assert P.load_library().spqr_packed_bytes(64, 64, 3, 4, 3, 16, 16, 0) == -3
    assert P.load_library().spqr_packed_bytes(64, 64, 3, 3, 3, 16, 8, 0) == -3
    assert P.load_library().spqr_packed_bytes(60, 64, 3, 3, 3, 16, 16, 0) == -2
    assert P.load_library().spqr_packed_bytes(64, 1 << 17, 3, 3, 3, 16, 16, 0) == -2
    assert "NULL" in P.spqr_strerror(-1)


@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", [
    (3, 16, 16, 1, 2, 3), (3, 16, 16, 0, 3, 70), (4, 16, 16, 1, 2, 130), (4, 16, 16, 0, 1, 64),
    (3, 8, 32, 1, 3, 65), (3, 8, 32, 0, 2, 129), (3, 16, 32, 0, 2, 5), (4, 32, 64, 1, 2, 3),
])
def test_pack_round_trip_through_independent_reader(w, b1, b2, axis, ntr, ntc):
    tr, tc = synth.tile_shape(b1, b2, axis)
    f = synth.make_matrix(ntr * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis,
                          outlier_rate=0.0, seed=(21, w, b1, b2, axis))
    buf = P.pack_host(f)
    got = layout_reader.read_packed(buf, f.m, f.n, w, b1, b2, axis)
    assert np.array_equal(got["Q"], f.Q)
    assert np.array_equal(got["s_q"], f.s_q)
    assert np.array_equal(got["z_q"], f.z_q)
    for k in ("s_s", "z_s", "s_z", "z_z"):
        assert np.array_equal(got[k].view(np.uint16), getattr(f, k).view(np.uint16)), k


@pytest.mark.parametrize("layout,lv", [("round_zero", 2), ("stats16", 3)])
@pytest.mark.parametrize("w,b1,b2,axis,ntr,ntc", [
    (3, 16, 16, 1, 2, 3), (3, 16, 16, 0, 3, 70), (4, 16, 16, 1, 2, 130), (3, 8, 32, 1, 3, 65), (3, 8, 32, 0, 2, 129),
    (3, 48, 16, 0, 2, 5), (4, 32, 64, 1, 2, 3),
])
def test_variant_pack_round_trip_through_independent_reader(layout, lv, w, b1, b2, axis, ntr, ntc):
    tr, tc = synth.tile_shape(b1, b2, axis)
    f = synth.make_matrix(ntr * tr, ntc * tc, w_bits=w, beta1=b1, beta2=b2, group_axis=axis, outlier_rate=0.0,
                          seed=(22, w, b1, b2, axis), stat_layout=layout)
    got = layout_reader.read_packed(P.pack_host(f), f.m, f.n, w, b1, b2, axis, lv)
    assert np.array_equal(got["Q"], f.Q)
    if lv == 2:
        assert set(got) == {"Q", "s_q", "z_q", "s_s", "z_s"}
        keys = ("s_q", "z_q", "s_s", "z_s")
    else:
        assert set(got) == {"Q", "s16", "z16"}
        keys = ("s16", "z16")
    for k in keys:
        a, b = got[k], getattr(f, k)
        assert np.array_equal(a.view(np.uint16) if a.dtype == np.float16 else a,
                              b.view(np.uint16) if b.dtype == np.float16 else b), k


def test_packer_rejects_out_of_range_codes():
    f = synth.make_matrix(32, 32, outlier_rate=0.0)
    f.Q[3, 3] = 9
    with pytest.raises(P.SpQRError) as ei:
        P.pack_host(f)
    assert ei.value.status == -3


def test_host_side_descriptor_checks_need_no_gpu():
    # NULL descriptor and bad parameters are refused before any HIP call.
    lib = P.load_library()
    assert lib.spqr_gemv(None, None, None, 0, None) == -1
    d = P.binding.spqr_matrix_t()
    d.m = d.n = 64; d.w_bits = 7; d.s_bits = d.z_bits = 3; d.beta1 = d.beta2 = 16
    d.layout_version = 1
    assert lib.spqr_gemv(C.byref(d), None, None, 0, None) == -3
    d.w_bits = 3
    assert lib.spqr_gemv(C.byref(d), None, None, 0, None) == -1      # packed is NULL
    d.max_row_nnz = -5
    assert lib.spqr_gemv(C.byref(d), None, None, 0, None) == -3      # the hint is a count
    d.max_row_nnz = 0
    d.layout_version = 2
    assert lib.spqr_dequant_dense(C.byref(d), 0, None, None) == -1   # the integer zero-point layout: packed is NULL
    d.layout_version = 3
    assert lib.spqr_dequant_dense(C.byref(d), 0, None, None) == -3   # 16-bit statistics need s_bits = z_bits = 16
    d.layout_version = 4
    assert lib.spqr_dequant_dense(C.byref(d), 0, None, None) == -3


def _schedule_length(groups, nsteps, s, slots, nlong):
    """The launch plan's schedule, written out: workgroups in grid order, each on the place that is free first."""
    import heapq
    nsplit = -(-nsteps // s)
    free = [0.0] * slots
    end = 0.0
    for y in range(nsplit):
        steps = min(s, nsteps - y * s)
        for count, cost in ((groups, 0.3 + steps), (nlong, 0.45 if y == 0 else 0.02)):
            for _ in range(count):
                t = heapq.heappop(free) + cost
                heapq.heappush(free, t)
                end = max(end, t)
    return end + 0.3 * nsplit


@pytest.mark.parametrize("groups,nsteps,slots1,slots,nlong", [
    (64, 4, 512, 512, 128), (172, 4, 768, 512, 128), (64, 11, 512, 512, 128), (104, 7, 512, 512, 128),
    (280, 7, 512, 512, 128), (104, 18, 512, 512, 128), (344, 4, 256, 256, 128), (128, 11, 256, 256, 128),
    (1, 1, 512, 512, 0), (3, 40, 512, 512, 1), (2000, 2, 512, 512, 0), (312, 7, 768, 512, 384)])
def test_batch_launch_plan_is_the_shortest_simulated_schedule(groups, nsteps, slots1, slots, nlong):
    lib = C.CDLL(P.library_path())
    assert lib.spqr_set_option(2, 0) == 0                                # SPQR_OPT_BATCH_STEPS: not pinned
    fn = lib.spqr_plan_batch_steps
    fn.restype = C.c_int
    fn.argtypes = [C.c_int] * 5
    got = fn(groups, nsteps, slots1, slots, nlong)
    assert 1 <= got <= nsteps
    cands = [s for s in range(1, nsteps + 1) if s <= 32 or s == nsteps]
    cost = {s: _schedule_length(groups, nsteps, s, slots1 if s == 1 else slots, nlong) for s in cands}
    best = min(cost.values())
    assert cost[got] <= best + 1e-6
    assert got == max(s for s in cands if cost[s] <= best + 1e-9)       # ties: fewer splits
    assert fn(groups, nsteps, slots1, slots, nlong) == got               # remembered, same answer


def test_batch_launch_plan_arguments_and_the_pinned_choice():
    lib = C.CDLL(P.library_path())
    fn = lib.spqr_plan_batch_steps
    fn.restype = C.c_int
    fn.argtypes = [C.c_int] * 5
    for bad in ((0, 4, 512, 512, 0), (4, 0, 512, 512, 0), (4, 4, 0, 512, 0), (4, 4, 512, 0, 0), (4, 4, 512, 512, -1)):
        assert fn(*bad) == -3                                            # SPQR_ERR_PARAM
    assert fn(100, 1, 512, 512, 0) == 1
    # one group: splitting buys parallelism, 9 steps never stay in one workgroup
    assert fn(1, 9, 512, 512, 0) < 9
    # far more groups than places and nothing to balance: whole strips per workgroup cost the fewest partial results
    assert fn(512 * 40, 3, 512, 512, 0) == 3
    try:
        assert lib.spqr_set_option(2, 2) == 0                            # SPQR_OPT_BATCH_STEPS
        assert fn(280, 7, 512, 512, 128) == 2
        assert lib.spqr_set_option(2, 50) == 0
        assert fn(280, 7, 512, 512, 128) == 7
    finally:
        assert lib.spqr_set_option(2, 0) == 0
    assert lib.spqr_set_option(2, -1) == -3 and lib.spqr_set_option(9, 0) == -3 and lib.spqr_set_option(0, 4) == -3
    assert lib.spqr_set_option(3, 96) == -3 and lib.spqr_set_option(3, 64) == 0 and lib.spqr_set_option(3, 0) == 0   # SPQR_OPT_DENSE_ROWS


# ---- plan of a grouped batch-1 launch (host arithmetic; the launcher checks the same invariants before it launches) ----

def _plan_grouped(ms, ns, hints, nnz, w, b1, b2, axis, layout, max_waves, slots, mf):
    lib = C.CDLL(P.library_path())
    fn = lib.spqr_plan_grouped
    fn.restype = C.c_int
    k = len(ms)
    I, L = C.c_int32 * k, C.c_int64 * k
    ent, nw, lds = (C.c_int32 * (7 * k))(), C.c_int32(), C.c_int64()
    rc = fn(k, I(*ms), I(*ns), I(*hints), L(*nnz), w, b1, b2, axis, layout, max_waves, slots, mf, ent, C.byref(nw), C.byref(lds))
    return rc, [tuple(ent[7 * j:7 * j + 7]) for j in range(max(rc, 0))], nw.value, lds.value


def _check_grouped_plan(entries, nw, lds, ms, ns, hints, tr, tc, max_waves):
    """What the kernel assumes of every table entry."""
    assert 1 <= nw <= max_waves and lds <= 160 * 1024
    assert len({e[0] for e in entries}) == len(entries)
    for idx, R, Pw, cap, shared, spare, wgs in entries:
        m, n = ms[idx], ns[idx]
        xbytes = (2 * n + 15) // 16 * 16
        assert R * Pw == nw and R * tr <= 64 and 1 <= Pw <= -(-(n // tc) // 64)
        assert 64 * nw <= cap <= 8 * 64 * nw                       # a chunk per thread at least, eight at most
        assert wgs == -(-(m // tr) // R)
        assert xbytes <= lds
        if shared:
            assert 32 * cap <= lds and xbytes + 32 * spare <= lds and spare <= cap
        else:
            assert xbytes + 32 * cap <= lds and spare == 0
    wide = [e for e in entries if ns[e[0]] > ns[0]]
    assert entries[:len(wide)] == wide                             # the wider matrices first in the grid
    assert all(e[4] == 1 for e in wide) and all(e[4] == 0 for e in entries[len(wide):])


def test_grouped_plan_of_the_65b_block_takes_down_along_with_its_products_over_x():
    ms, ns = [8192] * 4 + [22016] * 2 + [8192], [8192] * 6 + [22016]
    hints = [205, 204, 203, 202, 207, 201, 509]
    nnz = [int(0.02 * m * n) for m, n in zip(ms, ns)]
    rc, ent, nw, lds = _plan_grouped(ms, ns, hints, nnz, 3, 8, 32, 1, 1, 8, 12, 1)
    assert rc == 7 and nw == 4
    _check_grouped_plan(ent, nw, lds, ms, ns, hints, 8, 32, 8)
    down = ent[0]
    assert down[0] == 6 and down[1:3] == (2, 2) and down[4] == 1 and down[6] == 512
    assert 2 * 8 * 509 // 8 + 2 <= down[3]                         # by the hint, a workgroup's chunks fit one round
    assert all(e[1:3] == (4, 1) for e in ent[1:])                  # the six: four strips, one wavefront each
    assert 3 * (lds + 6144) <= 160 * 1024                          # three workgroups per compute unit still
    # without the hint on down's longest row it waits for a launch of its own; without outliers it needs none
    rc, ent, nw, lds = _plan_grouped(ms, ns, hints[:6] + [0], nnz, 3, 8, 32, 1, 1, 8, 12, 1)
    assert rc == 6 and all(e[0] != 6 for e in ent)
    rc, ent, nw, lds = _plan_grouped(ms, ns, hints[:6] + [0], nnz[:6] + [0], 3, 8, 32, 1, 1, 8, 12, 1)
    assert rc == 7 and ent[0][0] == 6 and ent[0][4] == 1


def test_grouped_plan_with_long_outlier_rows_depends_on_the_length_of_the_launch():
    # LLaMA-33B shapes, rows of up to n outliers: one strip per workgroup for down, rounds on the LDS behind x
    ms, ns = [6656] * 4 + [17920] * 2 + [6656], [6656] * 6 + [17920]
    nnz = [int(0.01 * m * n) for m, n in zip(ms, ns)]
    rc, ent, nw, lds = _plan_grouped(ms, ns, ns, nnz, 4, 16, 16, 1, 1, 8, 12, 0)
    assert rc == 7
    _check_grouped_plan(ent, nw, lds, ms, ns, ns, 16, 16, 8)
    assert ent[0][0] == 6 and ent[0][1:3] == (1, nw) and ent[0][4] == 1 and ent[0][5] >= 64 * nw
    # LLaMA-7B shapes: the whole block is long enough (2.3 steps per wavefront slot), q and down alone are not
    ms, ns = [4096] * 4 + [11008] * 2 + [4096], [4096] * 6 + [11008]
    nnz = [int(0.01 * m * n) for m, n in zip(ms, ns)]
    rc, ent, nw, lds = _plan_grouped(ms, ns, ns, nnz, 3, 16, 16, 1, 1, 16, 16, 0)
    assert rc == 7 and ent[0][0] == 6 and ent[0][1:3] == (1, nw)
    _check_grouped_plan(ent, nw, lds, ms, ns, ns, 16, 16, 16)
    rc, ent, nw, lds = _plan_grouped([4096, 4096], [4096, 11008], [4096, 11008], [167772, 450888], 3, 16, 16, 1, 1, 16, 16, 0)
    assert rc == 1 and ent[0][0] == 0
    # the same pair with short rows everywhere: together
    rc, ent, nw, lds = _plan_grouped([4096, 4096], [4096, 11008], [66, 145], [167772, 450888], 3, 16, 16, 1, 1, 16, 16, 0)
    assert rc == 2 and ent[0][0] == 1 and ent[0][4] == 1
    _check_grouped_plan(ent, nw, lds, [4096, 4096], [4096, 11008], [66, 145], 16, 16, 16)


@pytest.mark.parametrize("w,b1,b2,axis,tr,tc,max_waves,slots,mf", [
    (3, 8, 32, 1, 8, 32, 8, 12, 1), (4, 16, 16, 1, 16, 16, 8, 12, 0), (3, 16, 16, 0, 16, 16, 16, 16, 0),
    (3, 8, 32, 0, 32, 8, 8, 12, 0), (4, 8, 32, 0, 32, 8, 8, 8, 0)])
def test_grouped_plans_keep_the_kernels_invariants(w, b1, b2, axis, tr, tc, max_waves, slots, mf):
    rng = np.random.default_rng(7)
    for _ in range(200):
        k = int(rng.integers(1, 9))
        base_n = tc * int(rng.integers(20, 400))
        ns = [base_n] + [base_n if rng.random() < 0.5 else tc * int(rng.integers(20, 1500)) for _ in range(k - 1)]
        ns = [min(n, 65536 // tc * tc) for n in ns]
        ms = [tr * int(rng.integers(1, 3000)) for _ in range(k)]
        nnz = [int(rng.choice([0.0, 0.005, 0.02, 0.1]) * m * n) for m, n in zip(ms, ns)]
        hints = [0 if z == 0 else int(rng.choice([0, max(1, 2 * z // m), n])) for z, m, n in zip(nnz, ms, ns)]
        rc, ent, nw, lds = _plan_grouped(ms, ns, hints, nnz, w, b1, b2, axis, 1, max_waves, slots, mf)
        if rc < 0:
            assert rc == -3                                        # no plan (an x that does not fit the LDS)
            continue
        assert 1 <= rc <= k and any(e[0] == 0 for e in ent)        # the base matrix is always taken
        _check_grouped_plan(ent, nw, lds, ms, ns, hints, tr, tc, max_waves)
        for idx, R, Pw, cap, shared, spare, wgs in ent:
            if shared and nnz[idx]:
                assert hints[idx] > 0                              # never without a hint


def test_grouped_plan_arguments():
    lib = C.CDLL(P.library_path())
    fn = lib.spqr_plan_grouped
    fn.restype = C.c_int
    one32, one64 = (C.c_int32 * 1)(4096), (C.c_int64 * 1)(0)
    ent, nw, lds = (C.c_int32 * 7)(), C.c_int32(), C.c_int64()
    assert fn(1, one32, one32, one32, one64, 3, 16, 16, 1, 1, 16, 16, 0, ent, C.byref(nw), C.byref(lds)) == 1
    assert fn(0, one32, one32, one32, one64, 3, 16, 16, 1, 1, 16, 16, 0, ent, C.byref(nw), C.byref(lds)) == -3
    assert fn(1, one32, one32, one32, one64, 3, 16, 16, 1, 1, 0, 16, 0, ent, C.byref(nw), C.byref(lds)) == -3
    assert fn(1, None, one32, one32, one64, 3, 16, 16, 1, 1, 16, 16, 0, ent, C.byref(nw), C.byref(lds)) == -1
    assert fn(1, one32, one32, one32, one64, 5, 16, 16, 1, 1, 16, 16, 0, ent, C.byref(nw), C.byref(lds)) == -3   # w_bits

