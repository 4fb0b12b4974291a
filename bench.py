#!/usr/bin/env python3
"""Benchmark of the structured-spinner hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--quick]

A "step" is one pass of the whole hot path (load, three sign-flip + transform
rounds, epilogue, store) over one batch of the headline workload, i.e. one
call of the C ABI.  Inputs are seeded, synthetic and already resident in HBM
when the timed region starts.  Rank 0 prints ONE JSON line; the same line
carries the per-size sweep (n = 2^10 .. 2^20) and the five configurations.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# plain fp32 vector-ALU peak: 256 CUs x 4 SIMDs x 32 lanes per cycle x 2.4 GHz operations per second (one wave64
# instruction per two cycles and SIMD: the published 157.3 TFLOP/s counted as one operation per lane instead
# of the two of a fused multiply-add); packed fp32 forms are not used
VALU_PEAK_GOPS = 256 * 4 * 32 * 2.4

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic_bytes(workload, diagonals):
    """HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what
    the same counter reads for spinner_stream_copy of known size): the row of profiles/hbm_traffic.md for this
    workload and diagonal form, or None where no counter run has been made."""
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 7 and cells[0] == workload and cells[1] == diagonals:
                    return int(cells[6].replace(" ", ""))
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_calls(torch, fn, steps, warmup):
    """Returns (wall ms per step, HIP-event ms per step) for `steps` back-to-back calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def time_graph(torch, fn, calls_per_graph, replays):
    """ms per call when `calls_per_graph` calls of fn are captured once into a HIP graph and replayed: what a
    launch-bound loop costs without the per-call host work.  The replayed result is what eager calls produce
    (fn writes the same outputs either way)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(calls_per_graph):
            fn()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * calls_per_graph)


def make_runner(torch, b, W, w, dev, diagonals):
    """Allocate inputs/outputs for workload w and return the callable that runs one step.

    diagonals = "signs": the +-1 diagonals are packed once, off the clock, into sign words
    (spinner_pack_signs) and the step calls spinner_apply_signs / spinner_hash_signs;
    diagonals = "fp32": the step calls spinner_apply / spinner_hash with the fp32 diagonals."""
    x = W.make_x_torch(w, dev)
    ds = torch.from_numpy(W.diag_sets(w)).to(dev)
    signs = b.spinner_pack_signs(ds) if diagonals == "signs" else None
    if w.kind == "hash":
        out = torch.empty((w.batch, w.L), dtype=torch.int32, device=dev)
        if signs is not None:
            def fn():
                b.spinner_hash_signs(x, signs, w.L, out_idx=out)
        else:
            def fn():
                b.spinner_hash(x, ds, out_idx=out)
    elif w.kind == "blocks":
        # stacked independent blocks: fp32 diagonals [L][3][n], one call
        width = (2 if w.epilogue == "cossin" else 1) * w.L * w.m
        out = torch.empty((w.batch, width), dtype=torch.float32, device=dev)

        def fn():
            b.spinner_apply_blocks(x, ds, w.m, w.epilogue, w.scale, out=out)
    elif w.kind == "codes":
        out = torch.empty((w.batch, w.m // 64), dtype=torch.int64, device=dev)
        need = b.spinner_codes_workspace_bytes(w.n, w.batch)
        ws = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
        d1, d2, d3 = ds[0, 0], ds[0, 1], ds[0, 2]
        if signs is not None:
            def fn():
                b.spinner_sign_codes_signs(x, signs, w.m, codes=out, workspace=ws)
        else:
            def fn():
                b.spinner_sign_codes(x, d1, d2, d3, w.m, codes=out, workspace=ws)
    else:
        width = 2 * w.m if w.epilogue == "cossin" else w.m
        out = torch.empty((w.batch, width), dtype=torch.float32, device=dev)
        need = b.spinner_workspace_bytes(w.n, w.batch, w.m, w.epilogue)
        ws = torch.empty(need, dtype=torch.uint8, device=dev) if need else None
        d1, d2, d3 = ds[0, 0], ds[0, 1], ds[0, 2]
        if signs is not None:
            def fn():
                b.spinner_apply_signs(x, signs, w.m, w.epilogue, w.scale, out=out, workspace=ws)
        else:
            def fn():
                b.spinner_apply(x, d1, d2, d3, w.m, w.epilogue, w.scale, out=out, workspace=ws)
    return fn, x


def measure(torch, b, W, w, dev, steps, warmup, diagonals="signs", ramp_ms=0.0, graph=False):
    fn, x = make_runner(torch, b, W, w, dev, diagonals)
    if ramp_ms > 0:
        # untimed: let the clocks settle under this kernel's own load (the first ~10-20 ms of a
        # compute-heavy kernel after idle or after a pure copy run measurably slower)
        t_end = time.perf_counter() + ramp_ms * 1e-3
        while time.perf_counter() < t_end:
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
    wall_ms, ev_ms = time_calls(torch, fn, steps, warmup)
    graph_ms = time_graph(torch, fn, 20, 10) if graph else None
    alg = W.algorithmic_bytes_per_vector(w) * w.batch
    sched = W.schedule_bytes_per_vector(w) * w.batch
    ops = W.adds_per_vector(w) * w.batch
    res = {
        "workload": w.name, "n": w.n, "batch": w.batch, "m": w.m, "epilogue": w.epilogue, "L": w.L,
        "diagonals": diagonals,
        "ms_per_step": round(wall_ms, 5), "kernel_ms": round(ev_ms, 5),
        "vectors_per_s": w.batch / (wall_ms * 1e-3),
        "algorithmic_bytes": alg,
        "achieved_GBs": alg / (ev_ms * 1e-3) / 1e9,
        "hbm_frac": alg / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        # what the kernels themselves read and write (memory-side cache + HBM): differs from the algorithmic
        # bytes only above the fused range, where the four-pass schedule moves a vector four times
        "schedule_bytes": sched,
        "schedule_GBs": sched / (ev_ms * 1e-3) / 1e9,
        "butterfly_adds_Gops": ops / (ev_ms * 1e-3) / 1e9,
        "valu_frac_adds_only": ops / (ev_ms * 1e-3) / 1e9 / VALU_PEAK_GOPS,
        "graph_ms_per_step": None if graph_ms is None else round(graph_ms, 5),
    }
    del fn, x
    torch.cuda.empty_cache()
    return res


def measure_gram(torch, b, dev, rows, m, steps, warmup):
    """Hamming Gram matrix of `rows` x `rows` random codes of m bits: pairs/s, and the fp4 operations per second of
    the inner-product table behind it (2 m per pair, on the matrix pipe) against the 10.1 PFLOP/s dense fp4 MFMA peak."""
    codes = torch.randint(-2**62, 2**62, (rows, m // 64), dtype=torch.int64, device=dev)
    out = torch.empty((rows, rows), dtype=torch.float32, device=dev)
    fn = lambda: b.spinner_angular_gram(codes, codes, m, out=out)
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    _, ev_ms = time_calls(torch, fn, steps, warmup)
    pairs = rows * rows
    res = {"workload": "angular_gram_%dx%d_m%d" % (rows, rows, m), "ms": round(ev_ms, 4),
           "pairs_per_s": pairs / (ev_ms * 1e-3),
           "fp4_TFLOPs": pairs * 2.0 * m / (ev_ms * 1e-3) / 1e12,
           "fp4_mfma_frac": pairs * 2.0 * m / (ev_ms * 1e-3) / 10.1e15}
    del codes, out
    torch.cuda.empty_cache()
    return res


def measure_layer(torch, b, dev, n, batch, steps, warmup, graph=False):
    """Adaptive layer: forward (keeps two activations) + backward (dx and the three diagonal gradients).
    Algorithmic bytes per element: forward 4 read + 12 written, backward 16 read + 4 written.
    graph=True also times the step as a captured HIP graph of 20 forward + backward pairs (launch-bound sizes)."""
    g = torch.Generator(device=dev)
    g.manual_seed(1610 + n)
    x = torch.randn((batch, n), generator=g, device=dev, dtype=torch.float32)
    dy = torch.randn((batch, n), generator=g, device=dev, dtype=torch.float32)
    d = 1.0 + 0.5 * torch.randn((3, n), generator=g, device=dev, dtype=torch.float32)
    y = torch.empty_like(x)
    dx = torch.empty_like(x)
    saved = torch.empty((2, batch, n), dtype=torch.float32, device=dev)
    dd = torch.empty((3, n), dtype=torch.float32, device=dev)
    ws = torch.empty(max(16, b.spinner_layer_workspace_bytes(n, batch)), dtype=torch.uint8, device=dev)
    fwd = lambda: b.spinner_layer_forward(x, d[0], d[1], d[2], 1.0, y=y, saved=saved)
    bwd = lambda: b.spinner_layer_backward(dy, x, saved, d[0], d[1], d[2], 1.0, dx=dx, dd=dd, workspace=ws)
    for _ in range(10):
        fwd(); bwd()
    torch.cuda.synchronize()
    _, f_ms = time_calls(torch, fwd, steps, warmup)
    _, b_ms = time_calls(torch, bwd, steps, warmup)
    wall_ms, _ = time_calls(torch, lambda: (fwd(), bwd()), steps, warmup)
    el = batch * n
    graph_ms = time_graph(torch, lambda: (fwd(), bwd()), 20, 10) if graph else None
    res = {"workload": "adaptive_layer_n%d_b%d" % (n, batch), "forward_ms": round(f_ms, 4), "backward_ms": round(b_ms, 4),
           "step_us_wall": round(wall_ms * 1e3, 2), "step_us_graph": None if graph_ms is None else round(graph_ms * 1e3, 2),
           "forward_GBs": round(16.0 * el / (f_ms * 1e-3) / 1e9, 1), "backward_GBs": round(20.0 * el / (b_ms * 1e-3) / 1e9, 1)}
    del x, dy, d, y, dx, saved, dd, ws
    torch.cuda.empty_cache()
    return res


def measure_sketch(torch, b, W, dev, n, d, m, steps, warmup, form):
    """Newton sketch: B = S diag(w) A and the d x d Gram matrix on the matrix pipe.  `form` names the path the library
    takes for this shape: the columns loaded as they lie (n <= 2^12, wide or small matrices), or transposition +
    projection + transposition."""
    import math as _m

    g = torch.Generator(device=dev)
    g.manual_seed(1610 + d)
    A = torch.randn((n, d), generator=g, device=dev, dtype=torch.float32)
    w = torch.rand(n, generator=g, device=dev, dtype=torch.float32) * 0.5
    ds = torch.from_numpy(W.rademacher_diagonals(n, 3, 77)).to(dev)
    Bm = torch.empty((m, d), dtype=torch.float32, device=dev)
    G = torch.empty((d, d), dtype=torch.float32, device=dev)
    ws = torch.empty(b.spinner_sketch_workspace_bytes(n, d, m), dtype=torch.uint8, device=dev)
    sk = lambda: b.spinner_sketch(A, w, ds[0], ds[1], ds[2], m, _m.sqrt(n / m), out=Bm, workspace=ws)
    gws = torch.empty(max(16, b.spinner_sketch_gram_workspace_bytes(m, d)), dtype=torch.uint8, device=dev)
    gr = lambda: b.spinner_sketch_gram(Bm, out=G, workspace=gws)
    for _ in range(10):
        sk(); gr()
    torch.cuda.synchronize()
    _, s_ms = time_calls(torch, sk, steps, warmup)
    _, g_ms = time_calls(torch, gr, steps, warmup)
    res = {"workload": "newton_sketch_n%d_d%d_m%d" % (n, d, m), "form": form, "sketch_ms": round(s_ms, 4), "gram_ms": round(g_ms, 4),
           # the method's own bytes: A read once, B written once
           "sketch_GBs": round((4.0 * n * d + 4.0 * m * d) / (s_ms * 1e-3) / 1e9, 1),
           "gram_TFLOPs": round(2.0 * m * d * d / (g_ms * 1e-3) / 1e12, 2), "gram_mfma_frac": round(2.0 * m * d * d / (g_ms * 1e-3) / 157.3e12, 4)}
    del A, w, ds, Bm, G, ws, gws
    torch.cuda.empty_cache()
    return res


def measure_struct(torch, b, dev, kind, n, batch, steps, warmup):
    """G_struct D2 H D1 member: Hadamard stages and FFT convolution of two vectors in LDS, one kernel; transforms beyond
    the LDS (n = 2^15, the largest size of the paper's timing table) through global memory with a workspace."""
    g = torch.Generator(device=dev)
    g.manual_seed(1610 + n)
    x = torch.randn((batch, n), generator=g, device=dev, dtype=torch.float32)
    d = (1.0 - 2.0 * torch.randint(0, 2, (2, n), generator=g, device=dev)).to(torch.float32)
    params = torch.randn(int(b.lib.spinner_struct_params(b.STRUCT_KINDS[kind], n)), generator=g, device=dev, dtype=torch.float32)
    spec = b.spinner_struct_prepare(kind, params, n)
    out = torch.empty((batch, n), dtype=torch.float32, device=dev)
    ws = torch.empty(max(16, b.spinner_struct_workspace_bytes(kind, n, batch)), dtype=torch.uint8, device=dev)
    fn = lambda: b.spinner_struct_apply_ws(x, kind, spec, d[0], d[1], n, 1.0, out=out, workspace=ws)
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    _, ms = time_calls(torch, fn, steps, warmup)
    res = {"workload": "struct_%s_n%d_b%d" % (kind, n, batch), "ms": round(ms, 4), "vectors_per_s": batch / (ms * 1e-3),
           "GBs_of_8B_per_element": round(8.0 * batch * n / (ms * 1e-3) / 1e9, 1)}
    del x, d, params, spec, out, ws
    torch.cuda.empty_cache()
    return res


def measure_feature_sizes(torch, b, W, dev):
    """Time per projected vector at the dimensions of the paper's feature-map timing table (2^9 .. 2^15) for the family
    members it lists: H D3 H D2 H D1 with the cos / sin feature map, and the G_struct D2 H D1 members (projection alone).
    2^24 input elements per call.  Context for that table, whose entries are CPU speed-ups over a dense product."""
    import math as _m

    rows = []
    for k in range(9, 16):
        n = 1 << k
        batch = (1 << 24) // n
        g = torch.Generator(device=dev)
        g.manual_seed(1610 + k)
        x = torch.randn((batch, n), generator=g, device=dev, dtype=torch.float32)
        ds = torch.from_numpy(W.rademacher_diagonals(n, 3, 90 + k)).to(dev)
        signs = b.spinner_pack_signs(ds[None].contiguous())
        out = torch.empty((batch, 2 * n), dtype=torch.float32, device=dev)
        ws = torch.empty(max(16, b.spinner_workspace_bytes(n, batch, n, "cossin")), dtype=torch.uint8, device=dev)
        fn = lambda: b.spinner_apply_signs(x, signs, n, "cossin", _m.sqrt(n), out=out, workspace=ws)
        _, ms = time_calls(torch, fn, 10, 5)
        row = {"n": n, "batch": batch, "hd3hd2hd1_features_ns_per_vector": round(ms * 1e6 / batch, 2)}
        outp = out[:, :n]
        for kind in ("circulant", "toeplitz", "skew_circulant"):
            params = torch.randn(int(b.lib.spinner_struct_params(b.STRUCT_KINDS[kind], n)), generator=g, device=dev, dtype=torch.float32)
            spec = b.spinner_struct_prepare(kind, params, n)
            so = torch.empty((batch, n), dtype=torch.float32, device=dev)
            sws = torch.empty(max(16, b.spinner_struct_workspace_bytes(kind, n, batch)), dtype=torch.uint8, device=dev)
            sfn = lambda: b.spinner_struct_apply_ws(x, kind, spec, ds[0], ds[1], n, 1.0, out=so, workspace=sws)
            _, sms = time_calls(torch, sfn, 10, 5)
            row["g_%s_ns_per_vector" % kind] = round(sms * 1e6 / batch, 2)
            del params, spec, so, sws
        rows.append(row)
        del x, ds, signs, out, outp, ws
        torch.cuda.empty_cache()
    return {"workload": "feature_table_sizes_2p9_2p15", "rows": rows}


def copy_ceiling(torch, b, dev, steps, warmup):
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(50):                      # bring the GPU out of its idle clocks before anything is timed
        b.spinner_stream_copy(src, dst)
    torch.cuda.synchronize()
    _, ev_ms = time_calls(torch, lambda: b.spinner_stream_copy(src, dst), steps, warmup)
    del src, dst
    torch.cuda.empty_cache()
    return 2 * 4 * (1 << 28) / (ev_ms * 1e-3) / 1e9


def cpu_baseline(W, w):
    """The oracle as it stands, timed on the host cores on a bounded sample of workload w."""
    import numpy as np

    from oracle import spinner_oracle as oracle

    oracle.build()
    per_vec_macs = 3.0 * w.n * w.n * w.L if w.n <= (1 << 14) else 3.0 * 2.0 * math.sqrt(w.n) * w.n
    sample = int(max(4, min(w.batch, 4096, 2.0e10 / per_vec_macs)))
    ws = W.Workload(w.name, w.kind, w.n, sample, w.m, w.epilogue, w.scale, w.L, w.dist, w.seed, sample)
    x = W.make_x_numpy(ws)
    ds = W.diag_sets(ws)
    oracle.hadamard_dense(16)          # load the library outside the timed region
    t0 = time.perf_counter()
    if w.kind == "hash":
        oracle.hash(x, ds)
    else:
        oracle.apply(x, ds[0, 0], ds[0, 1], ds[0, 2], w.m, w.epilogue, w.scale)
    dt = time.perf_counter() - t0
    return {"value": sample / dt, "unit": "vectors/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": "%d vectors of %s (n=%d), dense O(n^2) fp64 oracle, %.2f s wall" % (sample, w.name, w.n, dt)}


def cpu_fast_single_thread(W, w):
    """Context for the paper's own setting (Section 5: one CPU thread, a fast Hadamard routine): the same
    product by O(n log n) butterflies in numpy on one thread, on a small sample.  Not the oracle, not the product."""
    import numpy as np

    sample = int(max(8, min(w.batch, 2.0e8 / (w.n * math.log2(w.n)))))
    ws = W.Workload(w.name, w.kind, w.n, sample, w.m, w.epilogue, w.scale, w.L, w.dist, w.seed, sample)
    x = W.make_x_numpy(ws).astype(np.float32)
    ds = W.diag_sets(ws)[0]
    t0 = time.perf_counter()
    y = x
    for d in ds:
        y = y * d
        h = 1
        while h < w.n:                                   # one butterfly stage per index bit
            y = y.reshape(sample, w.n // (2 * h), 2, h)
            y = np.concatenate([y[:, :, :1] + y[:, :, 1:], y[:, :, :1] - y[:, :, 1:]], axis=2)
            h *= 2
        y = y.reshape(sample, w.n)
    y = y * np.float32(w.n ** -1.5)
    dt = time.perf_counter() - t0
    return {"value": sample / dt, "unit": "vectors/s", "cores": 1, "kind": "numpy butterflies, one thread",
            "sample": "%d vectors of %s (n=%d), %.2f s wall" % (sample, w.name, w.n, dt)}


def measure_next_rows(torch, b, W, dev, args):
    """The rows beyond the five configurations: sign codes and their Gram estimate, adaptive layer, Newton sketch,
    G_struct members, and the layer at the hidden sizes of the paper's MLP timing table."""
    nxt = []
    for name, w in W.NEXT.items():
        r = measure(torch, b, W, w, dev, max(3, args.steps // 2), max(2, args.warmup // 2), args.diagonals, ramp_ms=60.0)
        nxt.append({"workload": name, "ms": round(r["kernel_ms"], 4), "vectors_per_s": round(r["vectors_per_s"], 1),
                    "GBs": round(r["achieved_GBs"], 1), "hbm_frac": round(r["hbm_frac"], 4),
                    "valu_frac_adds_only": round(r["valu_frac_adds_only"], 4)})
        log("[bench] %s: %.4f ms  %.3e vec/s  %.0f GB/s (%.1f%%)  butterfly adds at %.1f%% of VALU peak" % (
            name, r["kernel_ms"], r["vectors_per_s"], r["achieved_GBs"], 100 * r["hbm_frac"],
            100 * r["valu_frac_adds_only"]))
    g = measure_gram(torch, b, dev, 16384, 4096, max(3, args.steps // 2), max(2, args.warmup // 2))
    log("[bench] %s: %.4f ms  %.3e pairs/s  %.2f fp4 PFLOP/s (%.1f%% of the dense fp4 MFMA peak)" % (
        g["workload"], g["ms"], g["pairs_per_s"], g["fp4_TFLOPs"] / 1e3, 100 * g["fp4_mfma_frac"]))
    nxt.append(g)
    lay = measure_layer(torch, b, dev, 4096, 65536, max(3, args.steps // 2), max(2, args.warmup // 2))
    log("[bench] %s: forward %.4f ms (%.0f GB/s), backward %.4f ms (%.0f GB/s)" % (
        lay["workload"], lay["forward_ms"], lay["forward_GBs"], lay["backward_ms"], lay["backward_GBs"]))
    nxt.append(lay)
    for shape in ((1 << 16, 512, 2048, "transposition + projection + transposition"),
                  (1 << 12, 4096, 2048, "columns loaded as they lie")):
        skt = measure_sketch(torch, b, W, dev, shape[0], shape[1], shape[2], 10, 3, shape[3])
        log("[bench] %s (%s): sketch %.4f ms (%.0f GB/s of its own bytes), Gram %.4f ms (%.1f TFLOP/s fp32 MFMA)" % (
            skt["workload"], skt["form"], skt["sketch_ms"], skt["sketch_GBs"], skt["gram_ms"], skt["gram_TFLOPs"]))
        nxt.append(skt)
    for kind, sn, sbatch in (("circulant", 4096, 16384), ("toeplitz", 4096, 16384), ("circulant", 1 << 15, 2048), ("toeplitz", 1 << 15, 2048)):
        st = measure_struct(torch, b, dev, kind, sn, sbatch, 5, 2)
        log("[bench] %s: %.4f ms  %.3e vec/s  (%.0f GB/s counting 8 B per element)" % (
            st["workload"], st["ms"], st["vectors_per_s"], st["GBs_of_8B_per_element"]))
        nxt.append(st)
    ft = measure_feature_sizes(torch, b, W, dev)
    log("[bench] ns per vector at n = 2^9..2^15, HD3HD2HD1 features / G_circ / G_Toeplitz / G_skew-circ: " + "  ".join(
        "%d: %.1f/%.1f/%.1f/%.1f" % (r["n"], r["hd3hd2hd1_features_ns_per_vector"], r["g_circulant_ns_per_vector"],
                                     r["g_toeplitz_ns_per_vector"], r["g_skew_circulant_ns_per_vector"]) for r in ft["rows"]))
    nxt.append(ft)
    # hidden sizes of the paper's MLP timing table (Table 2), one layer, batch 1024: forward + backward per step
    tbl = []
    for k in range(4, 13):
        r = measure_layer(torch, b, dev, 1 << k, 1024, 20, 5, graph=True)
        tbl.append({"h": 1 << k, "step_us_wall": r["step_us_wall"], "step_us_graph": r["step_us_graph"],
                    "kernels_us": round((r["forward_ms"] + r["backward_ms"]) * 1e3, 2)})
    log("[bench] adaptive layer, batch 1024, h=2^4..2^12, forward+backward us per step, eager wall / captured graph: " +
        " ".join("%.1f/%.1f" % (t["step_us_wall"], t["step_us_graph"]) for t in tbl))
    nxt.append({"workload": "adaptive_layer_table2_sizes_b1024", "rows": tbl})
    return nxt


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="sweep_plain_n2p12",
                    help="headline workload: sweep_plain_n2pK (K=10..20) or one of the cfg names")
    ap.add_argument("--diagonals", choices=["signs", "fp32"], default="signs",
                    help="how the +-1 diagonals reach the kernels: packed sign words prepared in advance "
                         "(spinner_*_signs) or fp32 arrays (spinner_apply / spinner_hash)")
    ap.add_argument("--quick", action="store_true", help="headline only: no sweep, no configs, no CPU baseline")
    ap.add_argument("--only", action="store_true", help="headline only, and a single JSON line without extras")
    ap.add_argument("--next-only", action="store_true",
                    help="only the rows beyond the five configurations (for profiling them); prints their JSON and exits")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards over the batch: vectors are independent, "
              "no collective is involved); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1610_06209_amd import binding as b
    from paper_1610_06209_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def resolve(name):
        if name in W.CONFIGS:
            return W.CONFIGS[name]
        if name in W.NEXT:
            return W.NEXT[name]
        if name.startswith("sweep_plain_n2p"):
            return W.sweep_workload(int(name[len("sweep_plain_n2p"):]))
        raise SystemExit("unknown workload %r" % name)

    if args.next_only:
        print(json.dumps({"next_rows": measure_next_rows(torch, b, W, dev, args)}), flush=True)
        return
    head = resolve(args.workload)
    copy_gbs = round(copy_ceiling(torch, b, dev, 10, 3), 1)
    log("[bench] plain copy kernel (1 GiB read + 1 GiB write): %.0f GB/s" % copy_gbs)
    log("[bench] headline %s: n=%d batch=%d, diagonals as %s" % (head.name, head.n, head.batch, args.diagonals))
    hres = measure(torch, b, W, head, dev, args.steps, args.warmup, args.diagonals, ramp_ms=200.0)
    log("[bench] %s: %.4f ms/step, %.3e vectors/s, %.0f GB/s (%.1f%% of 8 TB/s)" % (
        head.name, hres["ms_per_step"], hres["vectors_per_s"], hres["achieved_GBs"], 100 * hres["hbm_frac"]))

    extras = {"copy_ceiling_GBs": copy_gbs, "headline_frac_of_copy": round(hres["achieved_GBs"] / copy_gbs, 4)}
    if not (args.quick or args.only):
        other = "fp32" if args.diagonals == "signs" else "signs"
        ores = measure(torch, b, W, head, dev, args.steps, args.warmup, other, ramp_ms=100.0)
        extras["headline_other_diagonal_form"] = {"diagonals": other, "vectors_per_s": ores["vectors_per_s"],
                                                  "kernel_ms": ores["kernel_ms"], "GBs": round(ores["achieved_GBs"], 1),
                                                  "hbm_frac": round(ores["hbm_frac"], 4)}
        log("[bench] %s with diagonals as %s: %.4f ms, %.0f GB/s (%.1f%%)" % (
            head.name, other, ores["kernel_ms"], ores["achieved_GBs"], 100 * ores["hbm_frac"]))
        sweep = []
        for k in range(10, 21):
            w = W.sweep_workload(k)
            r = measure(torch, b, W, w, dev, max(3, args.steps // 2), max(2, args.warmup // 2), args.diagonals, ramp_ms=60.0)
            rf = measure(torch, b, W, w, dev, max(3, args.steps // 2), max(2, args.warmup // 2), "fp32", ramp_ms=60.0)
            row = {"log2n": k, "batch": w.batch, "ms": round(r["kernel_ms"], 4),
                   "vectors_per_s": round(r["vectors_per_s"], 1), "GBs": round(r["achieved_GBs"], 1),
                   "hbm_frac": round(r["hbm_frac"], 4), "frac_of_copy": round(r["achieved_GBs"] / copy_gbs, 4),
                   "fp32_diag_ms": round(rf["kernel_ms"], 4), "fp32_diag_GBs": round(rf["achieved_GBs"], 1),
                   "fp32_diag_hbm_frac": round(rf["hbm_frac"], 4),
                   "traffic": measured_traffic_bytes(w.name, args.diagonals)}
            if r["schedule_bytes"] != r["algorithmic_bytes"]:
                # four passes: 32 B per element go through the memory-side cache and HBM together
                row["schedule_GBs_cache_and_hbm"] = round(r["schedule_GBs"], 1)
                row["fp32_diag_schedule_GBs_cache_and_hbm"] = round(rf["schedule_GBs"], 1)
            sweep.append(row)
            log("[bench] sweep n=2^%d batch=%d: %.4f ms  %.3e vec/s  %.0f GB/s (%.1f%%)   [fp32 diagonals: %.0f GB/s (%.1f%%)]%s" % (
                k, w.batch, r["kernel_ms"], r["vectors_per_s"], r["achieved_GBs"], 100 * r["hbm_frac"],
                rf["achieved_GBs"], 100 * rf["hbm_frac"],
                "" if r["schedule_bytes"] == r["algorithmic_bytes"] else
                "   four passes move %.0f GB/s through cache + HBM" % r["schedule_GBs"]))
        extras["sweep"] = sweep
        target = [t for t in sweep if 10 <= t["log2n"] <= 14]
        ws = min(target, key=lambda t: t["hbm_frac"])
        wf = min(target, key=lambda t: t["fp32_diag_hbm_frac"])
        extras["min_frac_2p10_2p14"] = {args.diagonals: {"frac": ws["hbm_frac"], "log2n": ws["log2n"]},
                                        "fp32": {"frac": wf["fp32_diag_hbm_frac"], "log2n": wf["log2n"]}}
        log("[bench] lowest fraction of the HBM peak over n = 2^10 .. 2^14: %s" % json.dumps(extras["min_frac_2p10_2p14"]))
        cfgs = []
        for name in W.CONFIG_ORDER:
            w = W.CONFIGS[name]
            # the smallest configuration is launch-bound: also time it as a captured HIP graph of 20 steps
            r = measure(torch, b, W, w, dev, max(3, args.steps // 2), max(2, args.warmup // 2), args.diagonals, ramp_ms=60.0,
                        graph=(w.batch * w.n <= (1 << 20)))
            cfgs.append({"workload": name, "ms": round(r["kernel_ms"], 4), "vectors_per_s": round(r["vectors_per_s"], 1),
                         "GBs": round(r["achieved_GBs"], 1), "hbm_frac": round(r["hbm_frac"], 4),
                         "frac_of_copy": round(r["achieved_GBs"] / copy_gbs, 4),
                         "valu_frac_adds_only": round(r["valu_frac_adds_only"], 4),
                         "traffic": measured_traffic_bytes(name, args.diagonals)})
            if r["schedule_bytes"] != r["algorithmic_bytes"]:
                cfgs[-1]["schedule_GBs_cache_and_hbm"] = round(r["schedule_GBs"], 1)
            if r["graph_ms_per_step"] is not None:
                cfgs[-1]["graph_ms_per_step"] = r["graph_ms_per_step"]
                log("[bench] %s as a HIP graph of 20 steps: %.5f ms per step" % (name, r["graph_ms_per_step"]))
            log("[bench] %s: %.4f ms  %.3e vec/s  %.0f GB/s (%.1f%%)  butterfly adds at %.1f%% of VALU peak" % (
                name, r["kernel_ms"], r["vectors_per_s"], r["achieved_GBs"], 100 * r["hbm_frac"],
                100 * r["valu_frac_adds_only"]))
        extras["configs"] = cfgs
        nxt = measure_next_rows(torch, b, W, dev, args)
        extras["next_rows"] = nxt

    traffic = measured_traffic_bytes(head.name, args.diagonals)
    alu_bound = head.kind in ("hash", "codes")
    line = {
        "metric": "HD3HD2HD1 vectors/s + achieved HBM GB/s vs peak, fp32, n=2^10..2^20",
        "value": hres["vectors_per_s"],
        "unit": "vectors/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": hres["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64" if head.epilogue == "cossin" and head.n <= (1 << 14) else "f32",
        "data": "synthetic",
        "config": {"workload": head.name, "n": head.n, "batch": head.batch, "m": head.m,
                   "epilogue": head.epilogue, "L": head.L,
                   "diagonals": "rademacher, " + ("packed sign words prepared off the clock" if args.diagonals == "signs"
                                                 else "fp32 arrays")},
        "roofline": {
            # hashing and sign codes write next to nothing and are bound by the plain fp32 vector ALU
            "bound": "alu" if alu_bound else "hbm",
            "achieved": hres["butterfly_adds_Gops"] / 1e3 if alu_bound else hres["achieved_GBs"],
            "peak": VALU_PEAK_GOPS / 1e3 if alu_bound else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if alu_bound else "GB/s",
            "frac": hres["valu_frac_adds_only"] if alu_bound else hres["hbm_frac"],
            "traffic": traffic,
            "kernel_ms": hres["kernel_ms"],
            "algorithmic_bytes": hres["algorithmic_bytes"],
        },
    }
    if "min_frac_2p10_2p14" in extras:
        # the target is stated for every n = 2^10 .. 2^14: the headline size is one of them, this is the worst
        line["roofline"]["min_frac_2p10_2p14"] = extras.pop("min_frac_2p10_2p14")
    if not (args.quick or args.only):
        line["cpu_baseline"] = cpu_baseline(W, head)
        log("[bench] cpu oracle: %.1f vectors/s on %d cores (%s)" % (
            line["cpu_baseline"]["value"], line["cpu_baseline"]["cores"], line["cpu_baseline"]["sample"]))
        if head.kind == "apply" and head.epilogue == "none" and head.m == head.n:
            line["cpu_fast_1thread"] = cpu_fast_single_thread(W, head)
            log("[bench] O(n log n) butterflies in numpy on one CPU thread: %.0f vectors/s (%s)" % (
                line["cpu_fast_1thread"]["value"], line["cpu_fast_1thread"]["sample"]))
    else:
        line["cpu_baseline"] = None
    line.update(extras)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
