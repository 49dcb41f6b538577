#!/usr/bin/env python3
"""Benchmark of the SpQR decode GEMV on one MI355X.

A step is one pass of the hot path over one batch of synthetic input: the seven
projections of one LLaMA-65B-shaped decoder block (configuration 4: q, k, v, o
8192x8192, gate, up 22016x8192, down 8192x22016; 3-bit codes, beta1=8, beta2=32,
2 % outliers of which 64 full columns), batch 1, each with its own input vector:
one spqr_gemv_grouped call (ONE launch: `down`, whose input is wider, rides
along in the grid of the six projections that read 8192 inputs; the launches
of a step are counted from a stream capture); --calls seven / fused issue them
as seven spqr_gemv calls or as four calls (q/k/v and gate/up through
spqr_gemv_fused).
Successive steps visit distinct copies of the weights (a pool larger than twice
the 256 MB last-level cache) so that every launch streams from HBM, and 60 GB of
other allocations stay resident beside them.  Launches are replayed from a HIP
graph on torch's current stream and timed with events on that stream; whole
sweeps over the pool are repeated until the timed region is at least 200 ms,
whatever --steps says, and the warm-up (200 ms of the same work at least) runs
into it without a pause: the figure is the sustained rate, past the 30-40 ms
after idle during which the chip runs slower (ms_per_step_by_quarter shows how
steady the timed region was).

Prints ONE JSON line (see the keys below).
"""
import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MIN_TIMED_MS = 200.0     # the timed region is never shorter than this
MIN_WARM_MS = 200.0      # nor is the warm-up that runs into it without a pause: for the first 30-40 ms of sustained load
                         # after idle the chip runs up to 35 % slower (launch durations under the tracer: 79 us, then
                         # 108, back to 80 within 30 ms), and what is reported is the sustained rate
MIN_SWEEP_MS = 20.0      # the same for every figure of the per-layer and per-block sweeps
SWEEPS_PER_GRAPH = 8     # passes over the pool of weight copies captured into the graph of the timed step


def measured_traffic(kernel_key):
    """HBM bytes per launch of the kernel, as read back from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
    command (each scaled by what the same counter reads for a copy of known size): the line
    `traffic_bytes_per_launch[<kernel_key>] = <bytes>` of a summary under profiles/.  None if no summary has it."""
    pat = re.compile(r"traffic_bytes_per_launch\[" + re.escape(kernel_key) + r"\]\s*=\s*([0-9]+)")
    pdir = os.path.join(ROOT, "profiles")
    try:
        names = sorted(os.listdir(pdir))
    except OSError:
        return None
    for nm in names:
        try:
            with open(os.path.join(pdir, nm), "r", encoding="utf-8", errors="replace") as fh:
                mt = pat.search(fh.read())
        except OSError:
            continue
        if mt:
            return int(mt.group(1))
    return None


def count_launches(torch, fn):
    """Kernel launches of `fn()`: the kernel nodes of a throw-away stream capture of it."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    st = torch.cuda.Stream()
    sp = C.c_void_p(st.cuda_stream)
    graph = C.c_void_p()
    with torch.cuda.stream(st):
        if hip.hipStreamBeginCapture(sp, C.c_int(2)) != 0:                # hipStreamCaptureModeRelaxed
            raise RuntimeError("hipStreamBeginCapture failed")
        try:
            fn()
        finally:
            rc = hip.hipStreamEndCapture(sp, C.byref(graph))
    if rc != 0 or not graph.value:
        raise RuntimeError("hipStreamEndCapture failed")
    n = C.c_size_t(0)
    hip.hipGraphGetNodes(graph, None, C.byref(n))
    nodes = (C.c_void_p * max(1, n.value))()
    hip.hipGraphGetNodes(graph, nodes, C.byref(n))
    kernels = 0
    for k in range(n.value):
        t = C.c_int(-1)
        hip.hipGraphNodeGetType(C.c_void_p(nodes[k]), C.byref(t))
        kernels += t.value == 0                                            # hipGraphNodeTypeKernel
    hip.hipGraphDestroy(graph)
    return kernels


def algorithmic_bytes(A, batch=1):
    """Bytes the method must move for one product: packed tiles + CSR + x + y (fp32)."""
    return A.compressed_bytes() + 2 * A.n * batch + 4 * A.m * batch


def time_layer(P, torch, A, X, copies, reps=6):
    """Simple timing: graph of one launch per weight copy, replayed `reps` times (batches of 4 and more: or streamed
    eagerly, whichever is faster)."""
    pool = [A] + [A.clone() for _ in range(copies - 1)]
    b = X.shape[0]
    Y = torch.empty((b, A.m), dtype=torch.float32, device=X.device)
    fn = (lambda M: P.spqr_gemv(M, X[0], out=Y[0])) if b == 1 else (lambda M: P.spqr_gemm_smallbatch(M, X, out=Y))
    for M in pool:
        fn(M)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for M in pool:
            fn(M)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    g.replay()
    torch.cuda.synchronize()
    e0.record(); g.replay(); e1.record()
    torch.cuda.synchronize()
    reps = max(reps, int(MIN_SWEEP_MS / max(e0.elapsed_time(e1), 1e-3)) + 1)   # a timed region of MIN_SWEEP_MS at least
    for _ in range(2 * reps):                # and twice that as warm-up running into it (see MIN_WARM_MS)
        g.replay()
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * copies)
    if b >= 4:
        # The batch path's scratch is an allocation node per call in a graph (about 10 us each on this runtime) but a
        # buffer the library keeps per stream for eager calls: eager streaming as well, the better of the two counts.
        for _ in range(2):
            e0.record()
            for _ in range(reps):
                for M in pool:
                    fn(M)
            e1.record()
            torch.cuda.synchronize()
            us = min(us, e0.elapsed_time(e1) * 1e3 / (reps * copies))
    return us


def time_block(P, torch, mats, x_h, x_f, copies, fused, reps=4):
    """One decoder block: q, k, v (input x_h), o (x_h), gate, up (x_h), down (x_f); x_h, x_f are vectors (batch 1)
    or [b, n] batches.  `mats` maps the layer name to a list of `copies` weight copies.  fused=True issues q/k/v
    and gate/up as one spqr_gemv_fused / spqr_gemm_fused call each (4 calls per block instead of 7)."""
    batch = x_h.dim() == 2
    shape = (lambda A: (x_h.shape[0], A.m)) if batch else (lambda A: (A.m,))
    ys = {nm: torch.empty(shape(ms[0]), dtype=torch.float32, device=x_h.device) for nm, ms in mats.items()}
    one = P.spqr_gemm_smallbatch if batch else P.spqr_gemv
    many = P.spqr_gemm_fused if batch else P.spqr_gemv_fused

    def block(c):
        if fused == "grouped":               # batch 1 only: every projection with its own input, one call
            names = ("q", "k", "v", "o", "gate", "up", "down")
            P.spqr_gemv_grouped([mats[nm][c] for nm in names], [x_f if nm == "down" else x_h for nm in names],
                                outs=[ys[nm] for nm in names])
            return
        if fused:
            many([mats[nm][c] for nm in ("q", "k", "v")], x_h, outs=[ys[nm] for nm in ("q", "k", "v")])
            one(mats["o"][c], x_h, out=ys["o"])
            many([mats[nm][c] for nm in ("gate", "up")], x_h, outs=[ys[nm] for nm in ("gate", "up")])
        else:
            for nm in ("q", "k", "v", "o", "gate", "up"):
                one(mats[nm][c], x_h, out=ys[nm])
        one(mats["down"][c], x_f, out=ys["down"])

    for c in range(copies):
        block(c)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    if batch:
        # batches are streamed eagerly: the library keeps fused batch calls out of captured graphs
        # (the first timed round still pays for the growth of the stream's memory pool: the better of two counts)
        reps *= 4
        best = None
        for _ in range(2):
            e0.record()
            for _ in range(reps):
                for c in range(copies):
                    block(c)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (reps * copies)
            best = us if best is None else min(best, us)
        return best
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for c in range(copies):
            block(c)
    g.replay()
    torch.cuda.synchronize()
    e0.record(); g.replay(); e1.record()
    torch.cuda.synchronize()
    reps = max(reps, int(MIN_SWEEP_MS / max(e0.elapsed_time(e1), 1e-3)) + 1)
    for _ in range(2 * reps):
        g.replay()
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * copies)


def run_block_sweep(rows, P, synth, torch, dev):
    """Whole decoder blocks of configurations 2-4 at batch 1 and 16, seven separate calls against four (q/k/v and
    gate/up fused)."""
    for cfg in (2, 3, 4):
        specs = synth.config_layers(cfg)
        mats, nbytes = {}, 0
        for li, sp in enumerate(specs):
            A = P.SpQRMatrix.from_logical(synth.make_config_layer(cfg, li, group_axis=1), dev)
            nbytes += algorithmic_bytes(A, 1)
            mats[sp.name] = [A]
        copies = max(3, int(512e6 // nbytes) + 1)
        for nm in mats:
            mats[nm] += [mats[nm][0].clone() for _ in range(copies - 1)]
        h, f = specs[0].n, specs[-1].n
        x_h = torch.from_numpy(synth.make_x(h, 1, seed=(cfg, 100))[0]).to(dev)
        x_f = torch.from_numpy(synth.make_x(f, 1, seed=(cfg, 101))[0]).to(dev)
        for b in (1, 16):
            if b > 1:
                x_h = torch.from_numpy(synth.make_x(h, b, seed=(cfg, 100))).to(dev)
                x_f = torch.from_numpy(synth.make_x(f, b, seed=(cfg, 101))).to(dev)
            for fused in (False, True) + (("grouped",) if b == 1 else ()):
                us = time_block(P, torch, mats, x_h, x_f, copies, fused)
                rows.append({"config": cfg, "layer": {False: "block(7 calls)", True: "block(q/k/v, gate/up fused: 4 calls)",
                                                      "grouped": "block(spqr_gemv_grouped: 1 call)"}[fused],
                             "m": 0, "n": 0, "w_bits": specs[0].w_bits, "beta1": specs[0].beta1, "beta2": specs[0].beta2,
                             "group_axis": 1, "batch": b, "outliers": f"{specs[0].outlier_rate:g} {specs[0].outlier_structure}",
                             "compressed_MB": round(nbytes / 1e6, 2), "us": round(us, 2),
                             "GBps": round(nbytes / us / 1e3, 1),
                             "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)})
        del mats
        torch.cuda.empty_cache()


def run_sweep(path, P, synth, torch, dev):
    rows = []
    for cfg in sorted(synth.CONFIGS):
        seen = set()
        for li, sp in enumerate(synth.config_layers(cfg)):
            if (sp.m, sp.n) in seen:
                continue
            seen.add((sp.m, sp.n))
            for axis in (1, 0):
                f = synth.make_config_layer(cfg, li, group_axis=axis)
                A = P.SpQRMatrix.from_logical(f, dev)
                del f
                copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
                for b in sp.batches:
                    X = torch.from_numpy(synth.make_x(sp.n, b, seed=(cfg, li, b))).to(dev)
                    us = time_layer(P, torch, A, X, copies)
                    nbytes = algorithmic_bytes(A, b)
                    rows.append({"config": cfg, "layer": sp.name, "m": sp.m, "n": sp.n, "w_bits": sp.w_bits,
                                 "beta1": sp.beta1, "beta2": sp.beta2, "group_axis": axis, "batch": b,
                                 "outliers": f"{sp.outlier_rate:g} {sp.outlier_structure}",
                                 "compressed_MB": round(nbytes / 1e6, 2), "us": round(us, 2),
                                 "GBps": round(nbytes / us / 1e3, 1),
                                 "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)})
                del A
                torch.cuda.empty_cache()
    # the statistic variants of the ablations (Sec. 5) on the largest and the headline-config shapes, batch 1
    for cfg, li in ((1, 0), (4, 0), (4, 4), (4, 6)):
        sp = synth.config_layers(cfg)[li]
        for lay in ("round_zero", "stats16"):
            A = P.SpQRMatrix.from_logical(synth.make_config_layer(cfg, li, group_axis=1, stat_layout=lay), dev)
            copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
            X = torch.from_numpy(synth.make_x(sp.n, 1, seed=(cfg, li, 1))).to(dev)
            us = time_layer(P, torch, A, X, copies)
            nbytes = algorithmic_bytes(A, 1)
            rows.append({"config": cfg, "layer": f"{sp.name} [{lay}]", "m": sp.m, "n": sp.n, "w_bits": sp.w_bits,
                         "beta1": sp.beta1, "beta2": sp.beta2, "group_axis": 1, "batch": 1,
                         "outliers": f"{sp.outlier_rate:g} {sp.outlier_structure}",
                         "compressed_MB": round(nbytes / 1e6, 2), "us": round(us, 2),
                         "GBps": round(nbytes / us / 1e3, 1),
                         "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)})
            del A
            torch.cuda.empty_cache()
    run_block_sweep(rows, P, synth, torch, dev)
    with open(path, "w") as fh:
        json.dump(rows, fh, indent=1)


def run_batch_probe(b, P, synth, torch, dev, axis):
    """spqr_gemm_smallbatch at batch b on every distinct layer of configuration 3: the library's choice of path
    against the vector path forced through spqr_set_option."""
    rows, seen = [], set()
    for li, sp in enumerate(synth.config_layers(3)):
        if (sp.m, sp.n) in seen:
            continue
        seen.add((sp.m, sp.n))
        f = synth.make_config_layer(3, li, group_axis=axis)
        A = P.SpQRMatrix.from_logical(f, dev)
        del f
        copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
        X = torch.from_numpy(synth.make_x(sp.n, b, seed=(3, li, b))).to(dev)
        us = time_layer(P, torch, A, X, copies)
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_VECTOR)
        us_vec = time_layer(P, torch, A, X, copies)
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_AUTO)
        nbytes = algorithmic_bytes(A, b)
        rows.append({"layer": sp.name, "m": sp.m, "n": sp.n, "batch": b, "us": round(us, 2),
                     "us_vector_path": round(us_vec, 2), "GBps": round(nbytes / us / 1e3, 1),
                     "dense_TFLOPs": round(2.0 * sp.m * sp.n * b / us / 1e6, 2)})
        del A
        torch.cuda.empty_cache()
    return rows

def run_batch_sweep(path, P, synth, torch, dev, axis):
    """Batches 2..16 on the distinct layers of configurations 2, 3 and 4: the vector kernel's slices of 4 against the
    matrix-core path (both forced through spqr_set_option) and the library's own choice; batches 32..256: the
    matrix-core slices of 16 against the dense-copy path.  The tables the rules in the library's dispatch are read
    from.  Written as JSON to `path`."""
    rows = []
    for cfg in (2, 3, 4):
        for li, sp in distinct_layers(synth, cfg):
            A = P.SpQRMatrix.from_logical(synth.make_config_layer(cfg, li, group_axis=axis), dev)
            copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
            for b in (2, 3, 4, 5, 6, 7, 8, 12, 16):
                X = torch.from_numpy(synth.make_x(sp.n, b, seed=(cfg, li, b))).to(dev)
                us = {}
                for nm, opt in (("auto", P.SPQR_BATCH_PATH_AUTO), ("vector", P.SPQR_BATCH_PATH_VECTOR),
                                ("matrix", P.SPQR_BATCH_PATH_MATRIX)):
                    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, opt)
                    us[nm] = round(time_layer(P, torch, A, X, copies), 2)
                P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_AUTO)
                rows.append({"config": cfg, "layer": sp.name, "m": sp.m, "n": sp.n, "batch": b, **us})
            # large batches: the slices of 16 against the dense-copy path
            for b in (32, 48, 64, 96, 128, 256):
                X = torch.from_numpy(synth.make_x(sp.n, b, seed=(cfg, li, b))).to(dev)
                us = {}
                for nm, opt in (("auto", P.SPQR_BATCH_PATH_AUTO), ("matrix", P.SPQR_BATCH_PATH_MATRIX),
                                ("dense", P.SPQR_BATCH_PATH_DENSE)):
                    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, opt)
                    us[nm] = round(time_layer(P, torch, A, X, min(copies, 3), reps=2), 2)
                P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_AUTO)
                rows.append({"config": cfg, "layer": sp.name, "m": sp.m, "n": sp.n, "batch": b, **us,
                             "auto_TFLOPs": round(2.0 * sp.m * sp.n * b / us["auto"] / 1e6, 1)})
            del A
            torch.cuda.empty_cache()
    with open(path, "w") as fh:
        json.dump(rows, fh, indent=1)


def distinct_layers(synth, cfg):
    seen, out = set(), []
    for li, sp in enumerate(synth.config_layers(cfg)):
        if (sp.m, sp.n) not in seen:
            seen.add((sp.m, sp.n))
            out.append((li, sp))
    return out


def run_batches(P, synth, torch, dev, axis):
    """Batches of 16 and 256 vectors on the distinct layers of configuration 3 (the library's choice of path:
    slices of 16 on the matrix cores, the dense-copy path at 256), same timing protocol as --sweep."""
    out = []
    for li, sp in distinct_layers(synth, 3):
        A = P.SpQRMatrix.from_logical(synth.make_config_layer(3, li, group_axis=axis), dev)
        copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
        for b in (16, 256):
            X = torch.from_numpy(synth.make_x(sp.n, b, seed=(3, li, b))).to(dev)
            us = time_layer(P, torch, A, X, copies, reps=3)
            out.append({"config": 3, "layer": sp.name, "m": sp.m, "n": sp.n, "batch": b, "us": round(us, 2),
                        "TFLOPs": round(2.0 * sp.m * sp.n * b / us / 1e6, 2)})
        del A
        torch.cuda.empty_cache()
    return out


def run_other_configs(P, synth, torch, dev, cfgs_axes):
    """Batch-1 figures of the other configurations' distinct layers (same protocol as --sweep, batch 1 only)."""
    out = []
    for cfg, axis in cfgs_axes:
        for li, sp in distinct_layers(synth, cfg):
            A = P.SpQRMatrix.from_logical(synth.make_config_layer(cfg, li, group_axis=axis), dev)
            copies = max(2, int(600e6 // A.compressed_bytes()) + 1)
            X = torch.from_numpy(synth.make_x(sp.n, 1, seed=(cfg, li, 1))).to(dev)
            us = time_layer(P, torch, A, X, copies)
            nbytes = algorithmic_bytes(A, 1)
            out.append({"config": cfg, "layer": sp.name, "m": sp.m, "n": sp.n, "w_bits": sp.w_bits, "beta1": sp.beta1,
                        "beta2": sp.beta2, "group_axis": axis, "compressed_MB": round(nbytes / 1e6, 2),
                        "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                        "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)})
            del A, X
            torch.cuda.empty_cache()
    return out


def run_other_blocks(P, synth, torch, dev, cfgs, axis):
    """Whole decoder blocks of the other configurations at batch 1: one spqr_gemv_grouped call per step (its launches
    counted from a stream capture), graph replay over distinct weight copies, warm-up running into the timed region."""
    out = []
    for cfg in cfgs:
        specs = synth.config_layers(cfg)
        base = [P.SpQRMatrix.from_logical(synth.make_config_layer(cfg, li, group_axis=axis), dev) for li in range(len(specs))]
        nbytes = sum(algorithmic_bytes(A, 1) for A in base)
        copies = max(3, int(600e6 // nbytes) + 1)
        pool = [base] + [[A.clone() for A in base] for _ in range(copies - 1)]
        xs = [torch.from_numpy(synth.make_x(sp.n, 1, seed=(cfg, li, 2))[0]).to(dev) for li, sp in enumerate(specs)]
        ys = [torch.empty(sp.m, dtype=torch.float32, device=dev) for sp in specs]
        P.spqr_gemv_grouped(pool[0], xs, outs=ys)
        torch.cuda.synchronize()
        launches = count_launches(torch, lambda: P.spqr_gemv_grouped(pool[0], xs, outs=ys))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in range(copies):
                P.spqr_gemv_grouped(pool[c], xs, outs=ys)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        g.replay()
        torch.cuda.synchronize()
        e0.record(); g.replay(); e1.record()
        torch.cuda.synchronize()
        reps = int(2 * MIN_SWEEP_MS / max(e0.elapsed_time(e1), 1e-3)) + 1
        for _ in range(2 * reps):
            g.replay()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (reps * copies)
        out.append({"config": cfg, "block": "q, k, v, o %dx%d + gate, up %dx%d + down %dx%d" % (
                        specs[0].m, specs[0].n, specs[4].m, specs[4].n, specs[6].m, specs[6].n),
                    "w_bits": specs[0].w_bits, "beta1": specs[0].beta1, "beta2": specs[0].beta2, "group_axis": axis,
                    "outliers": f"{specs[0].outlier_rate:g} {specs[0].outlier_structure}", "launches_per_step": launches,
                    "compressed_MB": round(nbytes / 1e6, 2), "us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                    "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)})
        del pool, base, g
        torch.cuda.empty_cache()
    return out


def run_encoder(torch, dev, with_cpu):
    """The quantiser (Alg. 1) on one 11008 x 4096 layer (the gate / up projection of configurations 1 and 2): H = 2 X X^T, its inverse factor, the sweep.  Inputs are drawn
    on the device from a seeded generator (W ~ N(0, 0.05^2) with 2 % of the entries six times larger, X = A G with
    A = I + 0.3 / sqrt(n) N(0, 1)); the first 64 rows (one workgroup of the sweep; rows of different tiles are
    independent) are re-run by the CPU oracle on the same H^ic and compared bit for bit, and that oracle run is the
    CPU baseline."""
    import numpy as np
    import paper_2306_03078_amd.encode_binding as E
    m, n, d = 11008, 4096, 4096; bits, b1, b2, tau, lam = 3, 16, 16, 20.0, 0.1
    gen = torch.Generator(device=dev); gen.manual_seed(1234)
    X = torch.randn(n, d, dtype=torch.float64, device=dev, generator=gen)
    A = torch.eye(n, dtype=torch.float64, device=dev) + 0.3 / n ** 0.5 * torch.randn(n, n, dtype=torch.float64, device=dev, generator=gen)
    X = A @ X
    W = 0.05 * torch.randn(m, n, dtype=torch.float64, device=dev, generator=gen)
    W[torch.rand(m, n, device=dev, generator=gen) < 0.02] *= 6
    del A

    def timed(fn, reps):
        fn(); torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            r = fn()
        b.record(); torch.cuda.synchronize()
        return r, a.elapsed_time(b) / reps
    H, t_h = timed(lambda: E.spqr_hessian(X), 3)
    ws = torch.empty(E._lib().spqr_inverse_cholesky_workspace_bytes(n), dtype=torch.uint8, device=dev)
    U, t_c = timed(lambda: E.spqr_inverse_cholesky(H, lam, workspace=ws), 3)
    del ws
    outs = E.spqr_quantize_device(W, U, bits, b1, b2, tau, want_final=False)
    wsq = outs.pop("workspace")
    _, t_q = timed(lambda: E.spqr_quantize_device(W, U, bits, b1, b2, tau, want_final=False, outputs=outs, workspace=wsq), 3)
    nnz = int(outs["row_ptr"][-1].item())
    ops = float(m) * n * n           # one product and one difference per weight and earlier column of its row
    res = {"workload": f"{m}x{n} layer, {d} calibration vectors, w={bits}, beta1={b1}, beta2={b2}, tau={tau}, lambda={lam}, "
                       "group_axis=0 (Alg. 1's orientation), binary64",
           "hessian_ms": round(t_h, 3), "hessian_TFLOPs": round(2.0 * n * n * d / t_h / 1e9, 2),
           "inverse_cholesky_ms": round(t_c, 3), "quantize_ms": round(t_q, 3),
           "weights_per_s": round(m * n / (t_q * 1e-3), 1), "outlier_rate": round(nnz / (m * n), 5),
           "roofline": {"bound": "alu", "kernel": "sweep_kernel<16>", "unit": "Tops/s",
                        "achieved": round(ops / (t_q * 1e-3) / 1e12, 3), "peak": 39.3,
                        "frac": round(ops / (t_q * 1e-3) / 1e12 / 39.3, 4),
                        "note": "binary64 products and differences of the error feedback, never fused (m n^2 of them); "
                                "peak = half the 78.6 TFLOP/s binary64 vector rate, which counts a fused multiply-add "
                                f"as two; the launch has m / 64 = {m // 64} workgroups for 256 compute units"}}
    if with_cpu:
        from oracle import spqr_encoder as enc
        rows = 64
        Wn = W[:rows].cpu().numpy(); Un = U.cpu().numpy()
        t = time.perf_counter()
        ref = enc.spqr_quantize(Wn, Un, bits, b1, b2, tau)
        dt = time.perf_counter() - t
        same = all(np.array_equal(outs[k][:rows].cpu().numpy().view(np.uint8) if outs[k].dtype == torch.uint8 else outs[k][:rows].cpu().numpy(),
                                  np.asarray(getattr(ref, k))) for k in ("Q", "s_q", "z_q"))
        same = same and np.array_equal(outs["outlier_mask"][:rows].cpu().numpy().astype(bool), ref.is_outlier)
        same = same and all(np.array_equal(outs[k][:rows // b2].cpu().numpy().view(np.uint16), np.asarray(getattr(ref, k)).view(np.uint16))
                            for k in ("s_s", "z_s", "s_z", "z_z"))
        assert same, "encoder parity failed on the timed buffers"
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        res["parity"] = f"rows 0..{rows - 1}: codes, statistic codes, second-level statistics and outlier mask bit-exact"
        res["cpu_baseline"] = {"value": round(rows * n / dt, 1), "unit": "weights/s", "cores": int(threads), "kind": "oracle",
                               "sample": f"the sweep on the first {rows} rows of the layer (H^ic given), {dt:.2f} s"}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=600)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--copies", type=int, default=3, help="distinct copies of the block's weights (470 MB each)")
    ap.add_argument("--group-axis", type=int, default=1)
    ap.add_argument("--filler-gb", type=int, default=60, help="other allocations kept resident beside the weights")
    ap.add_argument("--calls", choices=("grouped", "fused", "seven"), default="grouped",
                    help="how a step issues the seven projections: one spqr_gemv_grouped call, q/k/v and "
                         "gate/up as one spqr_gemv_fused call each (4 launches), or seven spqr_gemv calls")
    ap.add_argument("--block-config", type=int, choices=(2, 3, 4), default=4,
                    help="the configuration whose decoder block is the step (4, the headline workload, by default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-layer figures of configurations 0-3")
    ap.add_argument("--no-encoder", action="store_true", help="skip the timing of the quantiser (Alg. 1)")
    ap.add_argument("--encoder-only", action="store_true", help="time the quantiser (Alg. 1) alone and print its figures")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--sweep", metavar="PATH", default=None,
                    help="also time every distinct layer of all five configurations (both group orientations, "
                         "the batch sizes each configuration names) and write the table as JSON to PATH")
    ap.add_argument("--batch-probe", type=int, default=0, metavar="B",
                    help="also time spqr_gemm_smallbatch at batch B on the distinct layers of configuration 3, on the "
                         "path the library picks and on the vector path; adds \"batch_probe\" to the line")
    ap.add_argument("--batch-sweep", metavar="PATH", default=None,
                    help="also time batches 2..16 on the distinct layers of configurations 2-4 on the vector path, the "
                         "matrix-core path and the library's choice, and write the table as JSON to PATH")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run three 64 MiB device copies (a kernel of known traffic, for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2306_03078_amd as P
    import spqr_synth as synth

    P.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.encoder_only:
        print(json.dumps({"encoder": run_encoder(torch, dev, not args.no_cpu_baseline)}))
        return

    cfg = args.block_config
    specs = synth.config_layers(cfg)
    names = [sp.name for sp in specs]
    # 60 GB of other allocations stay resident while the block runs (sizing for 288 GB of HBM)
    filler = [torch.empty(6 * 1024 ** 3, dtype=torch.uint8, device=dev) for _ in range((args.filler_gb + 5) // 6)]
    for t in filler:
        t[:: 1 << 20].fill_(1)
    logical = [synth.make_config_layer(cfg, i, group_axis=args.group_axis) for i in range(len(specs))]
    base = [P.SpQRMatrix.from_logical(f, dev) for f in logical]
    for A in base:
        assert P.spqr_pack_check(A) == 0
    copies = max(2, args.copies)
    pool = [[A] + [A.clone() for _ in range(copies - 1)] for A in base]   # pool[layer][copy]
    h, ffn = specs[0].n, specs[-1].n
    x_h_np = synth.make_x(h, 1, seed=(cfg, 100))
    x_f_np = synth.make_x(ffn, 1, seed=(cfg, 101))
    x_h = torch.from_numpy(x_h_np[0]).to(dev)
    x_f = torch.from_numpy(x_f_np[0]).to(dev)
    xs = [x_f if sp.n == ffn else x_h for sp in specs]
    xs_np = [x_f_np if sp.n == ffn else x_h_np for sp in specs]
    ys = [torch.empty(f.m, dtype=torch.float32, device=dev) for f in logical]
    bytes_layer = [algorithmic_bytes(A) for A in base]
    step_bytes = sum(bytes_layer)
    pool_bytes = step_bytes * copies
    qkv = [i for i, nm in enumerate(names) if nm in ("q", "k", "v")]
    gu = [i for i, nm in enumerate(names) if nm in ("gate", "up")]
    rest = [i for i in range(len(names)) if i not in qkv and i not in gu]

    def run_step(k, calls):
        c = k % copies
        if calls == "grouped":
            P.spqr_gemv_grouped([pool[i][c] for i in range(len(base))], xs, outs=ys)
        elif calls == "fused":
            P.spqr_gemv_fused([pool[i][c] for i in qkv], x_h, outs=[ys[i] for i in qkv])
            P.spqr_gemv_fused([pool[i][c] for i in gu], x_h, outs=[ys[i] for i in gu])
            for i in rest:
                P.spqr_gemv(pool[i][c], xs[i], out=ys[i])
        else:
            for li in range(len(base)):
                P.spqr_gemv(pool[li][c], xs[li], out=ys[li])

    run_step(0, args.calls)
    torch.cuda.synchronize()
    launches_per_step = count_launches(torch, lambda: run_step(0, args.calls))
    stream = torch.cuda.current_stream()
    use_graph = not args.no_graph
    graph = None
    if use_graph:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            for k in range(copies):
                run_step(k, args.calls)
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):          # SWEEPS_PER_GRAPH passes over the pool per replay: the few us between
            for _ in range(SWEEPS_PER_GRAPH):  # two replays are shared by that many steps
                for k in range(copies):
                    run_step(k, args.calls)
    unit = SWEEPS_PER_GRAPH if graph is not None else 1     # sweeps come in units of this many

    def run_sweeps(nsweeps):                   # one sweep = one pass over the pool = `copies` steps
        assert nsweeps % unit == 0
        for _ in range(nsweeps // unit):
            if graph is not None:
                graph.replay()
            else:
                for k in range(copies):
                    run_step(k, args.calls)

    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    # two sweeps, then one that is timed to size the warm-up and the timed region
    run_sweeps(2 * unit)
    torch.cuda.synchronize()
    e0.record(); run_sweeps(unit); e1.record()
    torch.cuda.synchronize()
    est_ms_per_step = max(e0.elapsed_time(e1) / (unit * copies), 1e-3)
    # warm-up: at least the requested steps and MIN_WARM_MS of work; the timed region follows it on the stream
    # without a host synchronisation in between; it is cut into four windows to show how steady the rate is
    warm_sweeps = unit * math.ceil(max(args.warmup, MIN_WARM_MS / est_ms_per_step) / (unit * copies))
    nsweeps = 4 * unit * math.ceil(max(args.steps, MIN_TIMED_MS / est_ms_per_step) / (4 * unit * copies))
    steps_timed = nsweeps * copies
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    t0 = time.perf_counter()
    run_sweeps(warm_sweeps)
    marks[0].record()
    for w in range(4):
        run_sweeps(nsweeps // 4)
        marks[w + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * nsweeps / (nsweeps + warm_sweeps)
    e0, e1 = marks[0], marks[4]
    window_ms_per_step = [round(marks[w].elapsed_time(marks[w + 1]) / (steps_timed // 4), 6) for w in range(4)]
    ev_ms = e0.elapsed_time(e1)
    ms_per_step = ev_ms / steps_timed
    avg_launch_s = ev_ms * 1e-3 / (steps_timed * launches_per_step)
    gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    # the outputs of the last timed step (the last copy of every layer), for the parity check below
    got = [y.cpu().numpy().astype(np.float64) for y in ys]

    # per-layer figures: each layer alone, same pool rotation, a graph of one launch per copy
    per_layer = {}
    for li, sp in enumerate(specs):
        if any(v["m"] == sp.m and v["n"] == sp.n for v in per_layer.values()):
            continue
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in range(copies):
                P.spqr_gemv(pool[li][c], xs[li], out=ys[li])
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        reps = 200
        a.record()
        for _ in range(reps):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / (reps * copies)
        # isolated launches: one event pair around every single launch (eager), pool rotation as above
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(240)]
        for k, (p0, p1) in enumerate(pairs):
            p0.record()
            P.spqr_gemv(pool[li][k % copies], xs[li], out=ys[li])
            p1.record()
        torch.cuda.synchronize()
        iso = sorted(p0.elapsed_time(p1) * 1e3 for p0, p1 in pairs[40:])
        per_layer[sp.name] = {"m": sp.m, "n": sp.n, "us": round(us, 3),
                              "compressed_MB": round(bytes_layer[li] / 1e6, 3),
                              "GBps": round(bytes_layer[li] / (us * 1e-6) / 1e9, 1),
                              "frac_of_hbm_peak": round(bytes_layer[li] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                              "isolated_us": {"p10": round(iso[len(iso) // 10], 2), "median": round(iso[len(iso) // 2], 2),
                                              "p90": round(iso[9 * len(iso) // 10], 2)}}
    # the block issued the other ways
    other_us = {}
    for calls in ("grouped", "fused", "seven"):
        if calls == args.calls:
            continue
        other = torch.cuda.CUDAGraph()
        with torch.cuda.graph(other):
            for k in range(copies):
                run_step(k, calls)
        other.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(60):
            other.replay()
        e1.record()
        torch.cuda.synchronize()
        other_us["block_us_%s_calls" % calls] = round(e0.elapsed_time(e1) * 1e3 / (60 * copies), 2)
    del pool, graph, other
    torch.cuda.empty_cache()

    other_configs = batches = other_blocks = None
    if not args.no_configs:
        batches = run_batches(P, synth, torch, dev, args.group_axis)
        other_blocks = run_other_blocks(P, synth, torch, dev, [c for c in (2, 3) if c != cfg], args.group_axis)
        other_configs = run_other_configs(P, synth, torch, dev,
                                          [(0, args.group_axis), (1, args.group_axis), (2, args.group_axis),
                                           (3, args.group_axis), (4, 1 - args.group_axis)])

    encoder = None
    if not args.no_encoder and not args.no_configs:
        encoder = run_encoder(torch, dev, not args.no_cpu_baseline)

    if args.sweep:
        run_sweep(args.sweep, P, synth, torch, dev)

    if args.batch_sweep:
        run_batch_sweep(args.batch_sweep, P, synth, torch, dev, args.group_axis)

    batch_probe = None
    if args.batch_probe:
        batch_probe = run_batch_probe(args.batch_probe, P, synth, torch, dev, args.group_axis)

    if args.calibrate:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # Parity on the very buffers that were timed.  With the CPU baseline: the oracle's full decode + product of
    # every layer (the computation that is timed as the baseline) against the whole output vectors; without it:
    # sampled rows, computed by the oracle one by one.
    from oracle import spqr_oracle as orc
    cpu = None
    parity = []
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        t = time.perf_counter()
        refs = [orc.matvec(f, xs_np[li])[0] for li, f in enumerate(logical)]
        dt = time.perf_counter() - t
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        cpu = {"value": round(step_bytes / dt / 1e9, 4), "unit": "GB/s of compressed bytes", "cores": int(threads),
               "kind": "oracle",
               "sample": f"1 full step (all seven projections of the block at full size, once): fp64 decode to dense + "
                         f"outlier scatter + matvec, {dt:.2f} s; BLAS pool of {threads} threads, host shows "
                         f"{os.cpu_count()} logical cpus",
               "seconds_per_step": round(dt, 3), "us_per_layer": round(dt * 1e6 / len(base), 1)}
        for li in range(len(base)):
            parity.append(float(np.linalg.norm(got[li] - refs[li]) / np.linalg.norm(refs[li])))
        parity_kind = "whole output vectors"
    else:
        rng = np.random.default_rng(0)
        for li, f in enumerate(logical):
            rows = np.sort(rng.choice(f.m, size=64, replace=False))
            heavy = np.argsort(np.diff(f.row_ptr))[-4:]
            rows = np.unique(np.concatenate([rows, heavy]))
            ref = orc.matvec_rows(f, xs_np[li], rows)[0]
            parity.append(float(np.linalg.norm(got[li][rows] - ref) / np.linalg.norm(ref)))
        parity_kind = "sampled rows"
    assert max(parity) <= 1e-3, f"parity failed on the timed buffers: {parity}"

    sp0 = specs[0]
    tr, tc = synth.tile_shape(sp0.beta1, sp0.beta2, args.group_axis)
    tile = f"{tr},{tc}"
    kernel = ("gemv_tile256_%skernel<%d,%s,%d>" % ("" if args.calls == "seven" else "fused_", sp0.w_bits, tile, args.group_axis))
    kernel_key = "gemv_tile256_w%d_%s_axis%d_config%d_block" % (sp0.w_bits, tile.replace(",", "x"), args.group_axis, cfg)
    model = {2: "LLaMA-7B", 3: "LLaMA-33B", 4: "LLaMA-65B"}[cfg]
    shapes = {}
    for spx, nb in zip(specs, bytes_layer):
        shapes.setdefault((spx.m, spx.n), [0, nb])[0] += 1
    out = {
        "metric": "SpQR GEMV µs/layer + achieved HBM GB/s (% of peak), batch 1",
        "value": round(gbs, 2),
        "unit": "GB/s of compressed bytes (packed tiles + CSR + x + y) per second, whole step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "steps_timed": steps_timed, "timed_region_ms": round(ev_ms, 3),
        "warmup_steps_run": warm_sweeps * copies, "ms_per_step_by_quarter": window_ms_per_step,
        "ms_per_step": round(ms_per_step, 6),
        "us_per_layer": round(ms_per_step * 1e3 / len(base), 3),
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg}: one {model}-shaped decoder block, q/k/v/o {specs[0].m}x{specs[0].n} + gate/up "
                               f"{specs[4].m}x{specs[4].n} + down {specs[6].m}x{specs[6].n}, w={sp0.w_bits}, "
                               f"beta1={sp0.beta1}, beta2={sp0.beta2}, group_axis={args.group_axis}, "
                               f"{100 * sp0.outlier_rate:g}% outliers ({sp0.outlier_structure}), batch 1, beside "
                               f"{args.filler_gb} GB of filler allocations",
                   "launches_per_step": launches_per_step, "calls": args.calls, "weight_copies": copies,
                   "pool_MB": round(pool_bytes / 1e6, 1), "graph_replay": bool(use_graph), "steps_per_graph": unit * copies,
                   "wall_ms_per_step": round(wall * 1e3 / steps_timed, 6),
                   "parity_rel_l2": [float(f"{p:.3e}") for p in parity], "parity_checked_on": parity_kind},
        "layers": per_layer,
        **other_us,
        "roofline": {"bound": "hbm", "achieved": round(step_bytes / launches_per_step / avg_launch_s / 1e9, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(step_bytes / launches_per_step / avg_launch_s / 1e9 / HBM_PEAK_GBS, 4),
                     # the profile holds the one-launch block: no figure for another way of issuing the step
                     "traffic": measured_traffic(kernel_key) if args.calls == "grouped" and launches_per_step == 1 else None,
                     "kernel": kernel,
                     "algorithmic_bytes_per_launch": step_bytes // launches_per_step,
                     "avg_launch_us": round(avg_launch_s * 1e6, 3),
                     "note": "per launch = mean over the step's launches; the seven projections hold "
                             + ", ".join(f"{c} x {nb / 1e6:.1f} MB" for c, nb in shapes.values())
                             + " of algorithmic bytes; all launches run the same kernel body"},
        "cpu_baseline": cpu,
    }
    if other_configs is not None:
        out["other_configs_batch1"] = other_configs
        out["other_blocks_batch1"] = other_blocks
        out["batches_config3"] = batches
    if encoder is not None:
        out["encoder"] = encoder
    if batch_probe is not None:
        out["batch_probe"] = batch_probe
    print(json.dumps(out))


if __name__ == "__main__":
    main()
