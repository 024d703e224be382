"""Kernel-level measurements of the library on one MI355X.

    python -m paper_2412_20185_amd.microbench gemv     base GEMV kernel per shape: us, GB/s, fraction of 8 TB/s
    python -m paper_2412_20185_amd.microbench gemvshape  base GEMV launch shapes (waves per workgroup x groups per wave)
                                                       and the three ways of adding its K-slices
    python -m paper_2412_20185_amd.microbench selcost  cost of the exact selection: its own kernel, and inside the one-grid kernel
    python -m paper_2412_20185_amd.microbench fetch    residual fetch kernel per shape and number of wavefronts per column segment: us, GB/s
    python -m paper_2412_20185_amd.microbench ksweep   latency of a Llama-3-8B layer versus k (4-bit weights),
                                                       next to the knee model of the paper (Section 5.1)
    python -m paper_2412_20185_amd.microbench select   exact radix select versus the paper's approximate bucket
                                                       Top-K (Section 4.3): time per launch and recall
    python -m paper_2412_20185_amd.microbench rformats residual formats of the bit-width study (Table 2) at equal link
                                                       bytes: fetch kernel time and link rate for 2/4/8-bit and fp16 rows
    python -m paper_2412_20185_amd.microbench configs  decode-step latency on the two larger workloads: a Llama-3-70B-shaped
                                                       layer (3-bit codebook weights, fp16 residuals, k = 1 %) and a
                                                       32-layer Llama-3-8B-shaped step with 4-bit residuals at k_chunk = 15
    python -m paper_2412_20185_amd.microbench tune     the paper's parameter tuner (Section 4.4) on this GPU:
                                                       fetch workgroups and k_chunk per layer type for target slowdowns

Kernel durations are the dispatch timestamps the library records when
profiling is switched on (decdec_ws_set_profiling), i.e. what a kernel trace
reports.  Weights are random bytes in the packed layout (timing does not depend
on their values); several copies are rotated so that they come from HBM.
"""
from __future__ import annotations

import argparse
import json
import math
import sys

import numpy as np
import torch

from . import binding as B

HBM_PEAK_GBS = 8000.0
LINK_PEAK_GBS = 64.0

SHAPES_8B = [("q/o", 4096, 4096), ("k/v", 4096, 1024), ("gate/up", 4096, 14336), ("down", 14336, 4096),
             ("q+k+v", 4096, 6144), ("gate+up", 4096, 28672)]
SHAPES_70B = [("q/o", 8192, 8192), ("k/v", 8192, 1024), ("gate/up", 8192, 28672), ("down", 28672, 8192)]


def _operands(K, N, bits, wfmt, copies_bytes=600e6):
    d = B.Desc(K, N, bits, wfmt)
    nb = B.decdec_packed_bytes(d)
    copies = max(2, int(copies_bytes // nb) + 1)
    Wq = [torch.randint(0, 256, (nb,), dtype=torch.uint8, device="cuda") for _ in range(copies)]
    if wfmt == B.W_UNIFORM_G128:
        sc = torch.full((K // 128, N), 0.01, dtype=torch.float16, device="cuda")
        zl = torch.full((K // 128, N), 3.0, dtype=torch.float16, device="cuda")
        bytes_ = K * N * bits // 8 + 4 * N * (K // 128) + 2 * K + 2 * N
    else:
        sc = None
        zl = (torch.sort(torch.randn(N, 8, device="cuda"), dim=1).values * 0.02).half().contiguous()
        bytes_ = K * N * bits // 8 + 16 * N + 2 * K + 2 * N
    return d, Wq, sc, zl, bytes_


def gemv(args):
    ws = B.Workspace(28672, 28672, 16)
    print(f"{'model':4s} {'shape':8s} {'K':>6s} {'N':>6s} {'fmt':5s} {'MB':>8s} {'kernel us':>10s} {'GB/s':>8s} {'of 8TB/s':>9s}")
    for model, shapes in (("8B", SHAPES_8B), ("70B", SHAPES_70B)):
        for name, K, N in shapes:
            for bits, wfmt, tag in ((3, B.W_UNIFORM_G128, "u3"), (4, B.W_UNIFORM_G128, "u4"), (3, B.W_LUT_COL8, "lut3")):
                d, Wq, sc, zl, nbytes = _operands(K, N, bits, wfmt)
                x = torch.randn(K, device="cuda").half()
                y = torch.empty(N, dtype=torch.float16, device="cuda")
                for i in range(4):
                    B.decdec_gemv(d, x, Wq[i % len(Wq)], sc, zl, None, None, 0, y, ws)
                torch.cuda.synchronize()
                ws.set_profiling(args.reps)
                for i in range(args.reps):
                    B.decdec_gemv(d, x, Wq[i % len(Wq)], sc, zl, None, None, 0, y, ws)
                ms, n = ws.read_profile()["gemv"]
                ws.set_profiling(0)
                us = ms * 1e3 / n
                gbs = nbytes / us / 1e3
                print(f"{model:4s} {name:8s} {K:6d} {N:6d} {tag:5s} {nbytes / 1e6:8.2f} {us:10.2f} {gbs:8.0f} "
                      f"{gbs / HBM_PEAK_GBS:9.3f}", flush=True)
                del Wq
    ws.close()


def gemvshape(args):
    """Launch shapes of the base GEMV (k = 0): wavefronts per workgroup x groups of 128 input channels per
    wavefront, with the K-slices added by the accumulate kernel (acc), inside the kernel with one atomic per
    column and slice (ink) or not at all because one workgroup covers all of K (direct).  Kernel durations from the
    dispatch timestamps; call = wall time per call over HIP-graph replays of 16 back-to-back calls on
    rotating weight copies."""
    import time
    ws = B.Workspace(28672, 28672, 16)
    shapes = [("8B", n, K, N) for n, K, N in SHAPES_8B if n != "k/v"] + [("70B", n, K, N) for n, K, N in SHAPES_70B]
    fmts = {"u3": (3, B.W_UNIFORM_G128), "u4": (4, B.W_UNIFORM_G128), "lut3": (3, B.W_LUT_COL8)}
    stream = torch.cuda.Stream()
    print(f"{'model':4s} {'shape':8s} {'fmt':5s} {'waves':>5s} {'gpw':>4s} {'slices':>6s} {'sum':>7s} {'gemv us':>8s} "
          f"{'acc us':>7s} {'call us':>8s} {'GB/s(gemv)':>10s} {'GB/s(call)':>10s}")
    for model, name, K, N in shapes:
        G = K // 128
        for tag in args.fmts.split(","):
            bits, wfmt = fmts[tag]
            d, Wq, sc, zl, nbytes = _operands(K, N, bits, wfmt)
            x = torch.randn(K, device="cuda").half()
            y = torch.empty(N, dtype=torch.float16, device="cuda")
            combos = [(0, 0, 0)]
            for wpb in (4, 8, 16):
                for gpw in sorted({1, 2, 4, max(1, G // wpb), max(1, G // (2 * wpb)), max(1, G // (4 * wpb))}):
                    if gpw * wpb <= G or gpw == 1:
                        combos.append((wpb, gpw, 0))
                        if -(-G // (gpw * wpb)) > 1:
                            combos.append((wpb, gpw, 1))
            for wpb, gpw, ink in combos:
                ws.set_gemv_waves(wpb)
                ws.set_gemv_split(gpw)
                ws.set_inkernel_accumulate(bool(ink))
                for i in range(4):
                    B.decdec_gemv(d, x, Wq[i % len(Wq)], sc, zl, None, None, 0, y, ws)
                torch.cuda.synchronize()
                ws.set_profiling(args.reps)
                for i in range(args.reps):
                    B.decdec_gemv(d, x, Wq[i % len(Wq)], sc, zl, None, None, 0, y, ws)
                prof = ws.read_profile()
                ws.set_profiling(0)
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(16):
                        B.decdec_gemv(d, x, Wq[i % len(Wq)], sc, zl, None, None, 0, y, ws, stream)
                for _ in range(3):
                    g.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.reps):
                    g.replay()
                torch.cuda.synchronize()
                call_us = (time.perf_counter() - t0) * 1e6 / (16 * args.reps)
                del g
                us = prof["gemv"][0] * 1e3 / prof["gemv"][1]
                acc = prof["accumulate"][0] * 1e3 / max(prof["accumulate"][1], 1)
                eff_wpb = wpb or 4
                eff_gpw = gpw or max(1, -(-(N // 64) * G // 8192))
                slices = -(-G // (eff_gpw * eff_wpb))
                how = "direct" if slices == 1 else ("ink" if ink else "acc")
                print(f"{model:4s} {name:8s} {tag:5s} {wpb:5d} {gpw:4d} {slices:6d} {how:>7s} {us:8.2f} {acc:7.2f} "
                      f"{call_us:8.2f} {nbytes / us / 1e3:10.0f} {nbytes / call_us / 1e3:10.0f}", flush=True)
            del Wq
    ws.close()


def selcost(args):
    """What the exact selection costs where it runs: (a) the stand-alone selection kernel's duration, (b) the
    one-grid compensated kernel selecting for itself against the same kernel with the selection supplied
    (decdec_gemv_idx: its fetch workgroups read sc_indices from GPU memory instead of selecting).  3-bit
    weights, fp16 host residuals, N = 4096, activations N(0,1) with 0.5 % outlier channels."""
    import workloads
    from .layer import StoredLinear
    ws = B.Workspace(28672, 4096, 1024)
    print(f"{'K':>6s} {'k':>5s} {'select kernel us':>17s} {'fused, selects us':>18s} {'fused, supplied us':>19s} {'difference us':>14s}")
    for K in (4096, 8192, 14336, 28672):
        lin = StoredLinear.random(K, 4096, 3, B.W_UNIFORM_G128, 16, seed=K)
        xs = [torch.from_numpy(workloads.x_gauss_outliers(2, 0, 0, s, K)).cuda() for s in range(8)]
        y = torch.empty(4096, dtype=torch.float16, device="cuda")
        for frac in (0.001, 0.02):
            k = workloads.k_for_fraction(K, frac)
            idx = torch.empty(k, dtype=torch.int32, device="cuda")
            xsel = torch.empty(k, dtype=torch.float16, device="cuda")
            B.decdec_select_topk(xs[0], K, k, idx, xsel)
            res = {}
            for tag in ("select", "fused_selects", "fused_supplied"):
                ws.set_mode(B.MODE_SERIAL if tag == "select" else B.MODE_FUSED)
                ws.set_separate_select(tag == "select")
                run = ((lambda i: B.decdec_gemv_idx(lin.desc, xs[0], lin.Wq, lin.scales, lin.zeros, lin.R, None, k, idx, xsel, y, ws))
                       if tag == "fused_supplied" else (lambda i: lin.gemv(xs[i % 8], k, y, ws)))
                for i in range(4):
                    run(i)
                torch.cuda.synchronize()
                ws.set_profiling(args.reps)
                for i in range(args.reps):
                    run(i)
                prof = ws.read_profile()
                ws.set_profiling(0)
                ms, n = prof["select" if tag == "select" else "fetch"]
                res[tag] = ms * 1e3 / max(n, 1)
            print(f"{K:6d} {k:5d} {res['select']:17.2f} {res['fused_selects']:18.2f} {res['fused_supplied']:19.2f} "
                  f"{res['fused_selects'] - res['fused_supplied']:14.2f}", flush=True)
        del lin
    ws.close()


def fetch(args):
    ws = B.Workspace(28672, 28672, 4096)
    ws.set_mode(B.MODE_SERIAL)        # separate kernels, so that the fetch kernel's own duration is reported
    ws.set_separate_select(True)
    cases = [(4096, 1024, 81), (4096, 4096, 81), (4096, 6144, 81), (4096, 14336, 81), (14336, 4096, 286),
             (4096, 28672, 81), (4096, 4096, 512), (8192, 28672, 81), (28672, 8192, 286)]
    print("residual fetch kernel (fp16 rows, zero-copy): us / GB/s per number of wavefronts that share a column segment (0 = built-in choice)")
    for K, N, k in cases:
        d, Wq, sc, zl, _ = _operands(K, N, 3, B.W_UNIFORM_G128, copies_bytes=0)
        R = torch.empty((K, N), dtype=torch.float16, pin_memory=True)
        R.normal_(0, 0.003)
        xs = [torch.randn(K, device="cuda").half() for _ in range(8)]
        y = torch.empty(N, dtype=torch.float16, device="cuda")
        line = f"K {K:5d} N {N:5d} k {k:4d} ({k * N * 2 / 1e6:5.2f} MB):"
        for sp in (0, 2, 4, 8, 16, 32, 64, 128):
            ws.set_fetch_split(sp)
            for i in range(3):
                B.decdec_gemv(d, xs[i % 8], Wq[0], sc, zl, R, None, k, y, ws)
            torch.cuda.synchronize()
            ws.set_profiling(args.reps)
            for i in range(args.reps):
                B.decdec_gemv(d, xs[i % 8], Wq[0], sc, zl, R, None, k, y, ws)
            ms, n = ws.read_profile()["fetch"]
            ws.set_profiling(0)
            us = ms * 1e3 / n
            line += f"  s{sp}: {us:6.1f} / {k * N * 2 / us / 1e3:4.1f}"
        print(line, flush=True)
        del R
    ws.set_fetch_split(0)
    ws.close()


def rformats(args):
    """Table 2's design on the link: k_chunk channels per 1024 with 4-bit rows move as many bytes as
    2 k_chunk with 2-bit, k_chunk / 2 with 8-bit and k_chunk / 4 with fp16 rows.  Separate kernels
    (serial mode) so that the fetch kernel's own duration is what is reported."""
    ws = B.Workspace(28672, 28672, 8192)
    ws.set_mode(B.MODE_SERIAL)
    ws.set_separate_select(True)
    fmts = [("2-bit", B.R_INT2_SYM_COL, 2, 2.0), ("4-bit", B.R_INT4_SYM_COL, 4, 1.0),
            ("8-bit", B.R_INT8_SYM_COL, 8, 0.5), ("fp16", B.R_FP16, 16, 0.25)]
    print("fetch kernel at equal link bytes: us / GB/s over the link (rows) per residual format")
    print(f"{'K':>6s} {'N':>6s} {'k_chunk(4b)':>11s} {'MB':>6s}  " + "  ".join(f"{f[0]:>14s}" for f in fmts))
    for K, N in ((4096, 4096), (4096, 14336), (14336, 4096)):
        rows = {}
        for name, rfmt, bits, _ in fmts:
            R = torch.empty((K, N * bits // 8), dtype=torch.uint8, pin_memory=True)
            R.random_(0, 256)
            if bits == 16:  # keep fp16 payloads finite
                R.view(torch.float16).normal_(0, 0.003)
            rows[name] = R
        Rs = torch.full((N,), 1e-3, dtype=torch.float16, device="cuda")
        xs = [torch.randn(K, device="cuda").half() for _ in range(8)]
        y = torch.empty(N, dtype=torch.float16, device="cuda")
        for kc4 in (8, 32, 128):
            line = f"{K:6d} {N:6d} {kc4:11d} {kc4 * (K // 1024) * N / 2 / 1e6:6.2f}  "
            for name, rfmt, bits, mult in fmts:
                k = int(kc4 * mult) * (K // 1024)
                d = B.Desc(K, N, 3, B.W_UNIFORM_G128, rfmt)
                _, Wq, sc, zl, _ = _operands(K, N, 3, B.W_UNIFORM_G128, copies_bytes=0)
                scales = None if bits == 16 else Rs
                for i in range(3):
                    B.decdec_gemv(d, xs[i % 8], Wq[0], sc, zl, rows[name], scales, k, y, ws)
                torch.cuda.synchronize()
                ws.set_profiling(args.reps)
                for i in range(args.reps):
                    B.decdec_gemv(d, xs[i % 8], Wq[0], sc, zl, rows[name], scales, k, y, ws)
                ms, n = ws.read_profile()["fetch"]
                ws.set_profiling(0)
                us = ms * 1e3 / n
                nbytes = k * N * bits / 8
                line += f"  {us:7.1f} / {nbytes / us / 1e3:4.1f}"
            print(line, flush=True)
        del rows
    ws.close()


def configs(args):
    """Whole decode steps (every GEMV of every layer once) replayed as HIP graphs: wall time per step and
    per GEMV with compensation and without (k = 0), bytes over the host link and the link rate they imply."""
    import time
    import workloads
    from .layer import random_layer
    order = [("attn_in", ["q", "k", "v"]), ("o_in", ["o"]), ("mlp_in", ["gate", "up"]), ("down_in", ["down"])]
    cases = [
        ("Llama-3-70B-shaped layer, 3-bit codebook weights, fp16 residuals, k = 1 % of K, Student-t x",
         workloads.LLAMA3_70B_LAYER, 3, B.W_LUT_COL8, 16, 2, lambda K: workloads.k_for_fraction(K, 0.01), 4),
        ("32-layer Llama-3-8B-shaped step, 3-bit group-128 weights, 4-bit residuals, k_chunk = 15, Student-t x "
         "with 0.5 % outlier channels x30",
         workloads.LLAMA3_8B_LAYER, 3, B.W_UNIFORM_G128, 4, 32, lambda K: workloads.k_for_kchunk(K, 15), 5),
    ]
    for title, shapes, wbits, wfmt, rbits, nlayers, kof, cfg in cases:
        ys = {name: torch.empty(N, dtype=torch.float16, device="cuda") for name, _, N, _ in shapes}
        layers = [random_layer(shapes, wbits, wfmt, rbits, order, ys, seed=l) for l in range(nlayers)]
        Kof = {name: K for name, K, _, _ in shapes}
        inputs = sorted({(w, K) for _, K, _, w in shapes})
        extra = dict(outlier_frac=0.005, outlier_mult=30.0) if cfg == 5 else {}
        xpool = [{w: torch.from_numpy(workloads.x_student_t(cfg, 0, w, s, K, **extra)).cuda() for w, K in inputs}
                 for s in range(args.xpool)]
        ws = B.Workspace(max(K for _, K, _, _ in shapes), 2 * max(N for _, _, N, _ in shapes), 2048)
        stream = torch.cuda.Stream()
        res = {}
        for mode in ("compensated", "base"):
            def step(i):
                xs = xpool[i % args.xpool]
                for l in range(nlayers):
                    for (which, names), grp in zip(order, layers[l]):
                        B.decdec_gemv_multi(grp, xs[which], kof(Kof[names[0]]) if mode == "compensated" else 0, ws)
            graphs = []
            for i in range(args.xpool):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    step(i)
                graphs.append(g)
            nsteps = max(4, args.steps // nlayers)
            for i in range(2):
                graphs[i % len(graphs)].replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(nsteps):
                graphs[i % len(graphs)].replay()
            torch.cuda.synchronize()
            res[mode] = (time.perf_counter() - t0) * 1e6 / nsteps
            del graphs
        ngemv = nlayers * len(shapes)
        rbytes = nlayers * sum(kof(K) * N * rbits // 8 for _, K, N, _ in shapes)
        if wfmt == B.W_UNIFORM_G128:
            wbytes = nlayers * sum(K * N * wbits // 8 + 4 * N * (K // 128) + 2 * K + 2 * N for _, K, N, _ in shapes)
        else:
            wbytes = nlayers * sum(K * N * wbits // 8 + 16 * N + 2 * K + 2 * N for _, K, N, _ in shapes)
        print(title)
        print(f"  {ngemv} GEMVs per step; weights {wbytes / 1e6:.1f} MB, residual rows over the link {rbytes / 1e6:.2f} MB "
              f"({100 * rbytes / wbytes:.2f} % of the weight bytes)")
        print(f"  compensated: {res['compensated']:.1f} us per step, {res['compensated'] / ngemv:.2f} us per GEMV "
              f"(link {rbytes / res['compensated'] / 1e3:.1f} GB/s)")
        print(f"  base only  : {res['base']:.1f} us per step, {res['base'] / ngemv:.2f} us per GEMV "
              f"(HBM {wbytes / res['base'] / 1e3:.0f} GB/s); compensation adds "
              f"{100 * (res['compensated'] / res['base'] - 1):.1f} %", flush=True)
        ws.close()
        del layers, xpool


def ksweep(args):
    """Config-3 style: one Llama-3-8B-shaped layer, 4-bit weights, fp16 host
    residuals, k_chunk channels per 1024 input channels; activations redrawn
    each step.  Reports wall time per layer step (HIP-graph replay), per-kernel
    averages, and the paper's model t(k) = max(t_base, k N r/8 / BW_link)."""
    from .layer import LinearGroup, UniformLinear
    import workloads
    shapes = workloads.LLAMA3_8B_LAYER
    layers = []
    for l in range(args.layers):
        layers.append({name: UniformLinear(workloads.weights(3, l, name, K, N), 4) for name, K, N, _ in shapes})
    order = [("attn_in", ["q", "k", "v"]), ("o_in", ["o"]), ("mlp_in", ["gate", "up"]), ("down_in", ["down"])]
    ys = {name: torch.empty(N, dtype=torch.float16, device="cuda") for name, _, N, _ in shapes}
    groups = [[LinearGroup([lins[n] for n in names], [ys[n] for n in names]) for _, names in order] for lins in layers]
    Kof = {name: K for name, K, _, _ in shapes}
    inputs = sorted({(w, K) for _, K, _, w in shapes})
    xpool = [{w: torch.from_numpy(workloads.x_gauss_outliers(3, 0, w, s, K)).cuda() for w, K in inputs}
             for s in range(args.xpool)]
    ws = B.Workspace(14336, 28672, 2048)
    stream = torch.cuda.Stream()
    rows = []
    wbytes = sum(l.weight_bytes() for l in layers[0].values())
    for k_chunk in (0, 1, 2, 4, 8, 16, 32, 64, 128):
        def step(i):
            xs = xpool[i % args.xpool]
            for (which, names), grp in zip(order, groups[i % args.layers]):
                grp.gemv(xs[which], workloads.k_for_kchunk(Kof[names[0]], k_chunk), ws)
        graphs = {}
        period = math.lcm(args.layers, args.xpool)
        for i in range(period):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                step(i)
            graphs[i] = g
        for i in range(args.warmup):
            graphs[i % period].replay()
        torch.cuda.synchronize()
        import time
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % period].replay()
        torch.cuda.synchronize()
        us_step = (time.perf_counter() - t0) * 1e6 / args.steps
        ws.set_profiling(args.steps * len(order))
        for i in range(args.steps):
            step(i)
        prof = ws.read_profile()
        ws.set_profiling(0)
        rbytes = sum(workloads.k_for_kchunk(K, k_chunk) * N * 2 for _, K, N, _ in shapes)
        rows.append(dict(k_chunk=k_chunk, k_4096=workloads.k_for_kchunk(4096, k_chunk),
                         k_14336=workloads.k_for_kchunk(14336, k_chunk), us_per_layer=round(us_step, 1),
                         us_per_gemv=round(us_step / len(shapes), 2), residual_MB=round(rbytes / 1e6, 2),
                         gemv_us=round(prof["gemv"][0] * 1e3 / args.steps, 1),
                         select_us=round(prof["select"][0] * 1e3 / args.steps, 1),
                         fetch_us=round(prof["fetch"][0] * 1e3 / args.steps, 1),
                         accumulate_us=round(prof["accumulate"][0] * 1e3 / args.steps, 1),
                         link_GBs=round(rbytes / max(prof["fetch"][0], 1e-9) * args.steps / 1e6, 1) if k_chunk else 0.0))
        del graphs
    base = rows[0]["us_per_layer"]
    print(f"weights per layer {wbytes / 1e6:.1f} MB; columns: wall us per layer step (graph replay), per-kernel sums per "
          f"step (eager, kernel timestamps), model = max(base, residual bytes / 57.5 GB/s measured link ceiling)")
    print(f"{'k_chunk':>7s} {'k(4096)':>8s} {'k(14336)':>9s} {'resid MB':>9s} {'us/layer':>9s} {'us/GEMV':>8s} {'x base':>7s} "
          f"{'gemv':>7s} {'select':>7s} {'fetch':>7s} {'accum':>7s} {'link GB/s':>9s} {'model us':>9s}")
    for r in rows:
        model = max(base, r["residual_MB"] * 1e6 / 57.5e3)
        print(f"{r['k_chunk']:7d} {r['k_4096']:8d} {r['k_14336']:9d} {r['residual_MB']:9.2f} {r['us_per_layer']:9.1f} "
              f"{r['us_per_gemv']:8.2f} {r['us_per_layer'] / base:7.2f} {r['gemv_us']:7.1f} {r['select_us']:7.1f} "
              f"{r['fetch_us']:7.1f} {r['accumulate_us']:7.1f} {r['link_GBs']:9.1f} {model:9.1f}")
    # knee of the paper's model (Section 5.1) on this machine: k_chunk* = 1024 / R_bw * (b / r)
    r_bw = 8000.0 / 57.5
    print(f"paper's knee model with R_bw = 8000 / 57.5 = {r_bw:.0f}, 4-bit weights, fp16 residuals: "
          f"k_chunk* = 1024 / R_bw * (4 / 16) = {1024 / r_bw * 4 / 16:.2f}")
    print(json.dumps(rows))
    ws.close()


def select(args):
    """Stand-alone selection kernels on outlier-bearing activations (N(0,1), 0.5 % channels x U(10,50)):
    wall time per launch over back-to-back launches (run under rocprofv3 --kernel-trace --stats for the
    kernel durations) and recall of the approximate selector against the exact one (paper: about 80 % on
    real activations, Section 5.2).  Boundaries b0 / b15 are calibrated on 32 other draws (Section 4.3)."""
    import workloads
    print(f"{'K':>6s} {'k_chunk':>7s} {'k':>5s} {'exact us':>9s} {'bucket us':>10s} {'recall':>7s} {'b0':>8s} {'b15':>7s}")
    for K, which in ((4096, "attn_in"), (14336, "down_in")):
        for k_chunk in (8, 20, 32, 64, 128):
            k = k_chunk * K // 1024
            cal = torch.from_numpy(np.stack([workloads.x_gauss_outliers(3, 0, which, 1000 + s, K) for s in range(32)]))
            a = cal.float().abs()
            b0 = float(a.max())
            b15 = float(a.sort(dim=1).values[:, K - k].max())
            xs = [torch.from_numpy(workloads.x_gauss_outliers(3, 0, which, s, K)).cuda() for s in range(16)]
            ie = torch.empty(k, dtype=torch.int32, device="cuda")
            ib = torch.empty(k, dtype=torch.int32, device="cuda")
            v = torch.empty(k, dtype=torch.float16, device="cuda")
            rec = []
            for x in xs:
                B.decdec_select_topk(x, K, k, ie, v)
                B.decdec_select_bucket(x, K, k_chunk, b0, b15, ib, v)
                torch.cuda.synchronize()
                rec.append(np.intersect1d(ie.cpu().numpy(), ib.cpu().numpy()).size / k)
            times = []
            for fn in (lambda x: B.decdec_select_topk(x, K, k, ie, v),
                       lambda x: B.decdec_select_bucket(x, K, k_chunk, b0, b15, ib, v)):
                for i in range(20):
                    fn(xs[i % 16])
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(args.reps * 5):
                    fn(xs[i % 16])
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) * 1e3 / (args.reps * 5))
            print(f"{K:6d} {k_chunk:7d} {k:5d} {times[0]:9.2f} {times[1]:10.2f} {np.mean(rec):7.3f} {b0:8.2f} {b15:7.3f}",
                  flush=True)


class LayerHarness:
    """One decoder layer on the GPU plus measure(config) -> wall microseconds of its four calls replayed as a
    captured graph, for the parameter tuner (Section 4.4).  config: {type: (fetch workgroups per column
    segment, k_chunk)} over the layer types qkv, o, gu, d.  model "8b": Llama-3-8B shapes, 3-bit group-128
    weights quantised on the device from seeded N(0, 0.02^2) weights, fp16 host residuals; "70b": Llama-3-70B
    shapes with stored parameters drawn at random (3-bit codebook weights, fp16 host residuals)."""

    ORDER = [("qkv", "attn_in", ["q", "k", "v"]), ("o", "o_in", ["o"]), ("gu", "mlp_in", ["gate", "up"]),
             ("d", "down_in", ["down"])]

    def __init__(self, model: str = "8b", reps: int = 40, splits=(1, 2, 4, 8, 16, 32, 64)):
        import workloads
        from .layer import LinearGroup, StoredLinear, UniformLinear
        from . import tuner as T
        self.reps = reps
        shapes = workloads.LLAMA3_8B_LAYER if model == "8b" else workloads.LLAMA3_70B_LAYER
        if model == "8b":
            lins = {name: UniformLinear(workloads.weights(2, 0, name, K, N), 3) for name, K, N, _ in shapes}
            draw = lambda w, K: workloads.x_gauss_outliers(2, 0, w, 0, K)
        else:
            lins = {name: StoredLinear.random(K, N, 3, B.W_LUT_COL8, 16, seed=j) for j, (name, K, N, _) in enumerate(shapes)}
            draw = lambda w, K: workloads.x_student_t(4, 0, w, 0, K)
        ys = {name: torch.empty(N, dtype=torch.float16, device="cuda") for name, _, N, _ in shapes}
        self.groups = {t: LinearGroup([lins[n] for n in names], [ys[n] for n in names]) for t, _, names in self.ORDER}
        self.Kof = {t: lins[names[0]].K for t, _, names in self.ORDER}
        self.xin = {w: torch.from_numpy(draw(w, self.Kof[t])).cuda() for t, w, _ in self.ORDER}
        self.ws = B.Workspace(max(self.Kof.values()), 2 * max(l.N for l in lins.values()), 8192)
        self.stream = torch.cuda.Stream()
        self.types = [T.LayerType(t, self.Kof[t], sum(lins[n].N for n in names), candidates=tuple(splits))
                      for t, _, names in self.ORDER]
        self.cache = {}
        self.warm = False
        self.k_for_kchunk = workloads.k_for_kchunk

    def time_once(self, cfg) -> float:
        """Wall microseconds per layer of `cfg`, a fresh measurement."""
        import time
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=self.stream):
            for t, w, _ in self.ORDER:
                split, kc = cfg[t]
                self.ws.set_fetch_split(split)
                self.groups[t].gemv(self.xin[w], self.k_for_kchunk(self.Kof[t], kc), self.ws, self.stream)
        for _ in range(10 if self.warm else 200):   # the first measurement also brings the clocks up
            g.replay()
        self.warm = True
        best = float("inf")
        for _ in range(3):                          # timing noise is one-sided: the quickest of three batches
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(self.reps):
                g.replay()
            torch.cuda.synchronize()
            best = min(best, (time.perf_counter() - t0) * 1e6 / self.reps)
        return best

    def measure(self, cfg) -> float:
        """time_once, remembered per configuration (the tuner asks for the same one several times)."""
        key = tuple(sorted(cfg.items()))
        if key not in self.cache:
            self.cache[key] = self.time_once(cfg)
        return self.cache[key]

    def close(self):
        self.ws.set_fetch_split(0)
        self.ws.close()


def tune(args):
    """Section 4.4 on one decoder layer (--model 8b: Llama-3-8B shapes, 3-bit weights; 70b: Llama-3-70B shapes,
    3-bit codebook weights; fp16 host residuals): for each target slowdown over the uncompensated layer, the
    fetch workgroups per column segment (this library's counterpart of n_tb) and k_chunk per layer type.
    measure() = wall time of one layer (4 calls) replayed as a captured graph."""
    from . import tuner as T
    h = LayerHarness(args.model, reps=args.reps)
    print(f"model {args.model}")
    print("target   split cap  split (qkv,o,gu,d)   k_chunk (qkv,o,gu,d)   baseline us  tuned us  slowdown  frozen")
    for target in (0.025, 0.05, 0.1, 0.2, 0.5, 1.0, 2.0, 4.0):
        r = T.tune(h.types, h.measure, target, ntb_max_limit=64, k_chunk_limit=128)
        names = [t for t, _, _ in h.ORDER]
        print(f"{target * 100:6.1f}%  {r.ntb_max:9d}  {str(tuple(r.ntb[n] for n in names)):19s}  "
              f"{str(tuple(r.k_chunk[n] for n in names)):21s}  {r.baseline:11.1f}  {r.time:8.1f}  {r.slowdown * 100:7.1f}%  "
              f"{','.join(r.frozen) or '-'}", flush=True)
    print(f"{len(h.cache)} configurations measured")
    h.close()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=("gemv", "gemvshape", "selcost", "fetch", "ksweep", "select", "rformats", "configs", "tune"))
    ap.add_argument("--reps", type=int, default=40)
    ap.add_argument("--steps", type=int, default=96)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--xpool", type=int, default=8)
    ap.add_argument("--model", choices=("8b", "70b"), default="8b", help="tune: which layer shapes")
    ap.add_argument("--fmts", default="u3", help="gemvshape: comma-separated weight formats out of u3,u4,lut3")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    {"gemv": gemv, "gemvshape": gemvshape, "selcost": selcost, "fetch": fetch, "ksweep": ksweep, "select": select, "rformats": rformats, "configs": configs, "tune": tune}[args.what](args)
    return 0


if __name__ == "__main__":
    sys.exit(main())
