#!/usr/bin/env python3
"""Benchmark of the DETOX parameter-server step on one MI355X.

Workload the headline metric is quoted on: n = 45 nodes, r = 3, q = 5 Byzantine (ALIE attack),
d = 11,173,962 fp32 (ResNet-18-sized), synthetic and seeded.  One "step" is one pass of the whole
hot path over the resident n x d matrix:
    majority-vote filter -> 15 votes -> 5 block means -> Multi-Krum(f=1, m=3) -> d-vector.
The same run also times: every vanilla aggregator of the workload over all n rows; the other
aggregators on the same matrix; the two d = 25,000,000 workloads (n = 45 heavy-tailed, n = 105),
whose matrices are generated on the device with the same shapes and replication; the
mean-estimation setting; the dominant kernel on its own (HIP events inside the library); a
stream-read and an fp32-MFMA probe (the measured ceilings beside the published ones); and the CPU
oracle on the host cores.  Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
MFMA_F32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix, published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix, published peak


def measured_traffic(agg, n, d):
    """HBM bytes per launch of the dominant kernel as rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    measured them for this workload (the committed summary under profiles/, which also names the
    commit it was taken at), or (None, None)."""
    path = os.path.join(ROOT, "profiles", f"detox_step_{agg}__n{n}_d{d}.md")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\[.*\]: (\d+)", text, re.M)
    c = re.search(r"^measured_at_commit: (\S+)", text, re.M)
    return (int(m.group(1)) if m else None), (c.group(1) if c else None)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def traced_kernels(dx, fn, reps, np):
    """Mean duration (ms) of every kernel of `fn`, from the library's own HIP events on the launch stream."""
    with dx.trace() as tr:
        for _ in range(reps):
            fn()
        recs = tr.records()
    per = {}
    for name, ms in recs:
        per.setdefault(name, []).append(ms)
    return {k: float(np.mean(v)) for k, v in per.items()}


def probes(dx, torch, G):
    """Measured ceilings: stream read over the resident matrix's buffer, fp32 MFMA issue rate."""
    sink = torch.zeros(64, dtype=torch.float32, device=G.device)
    buf = G._base if G._base is not None else G
    nbytes = buf.numel() * 4
    ms, _ = time_steps(lambda: dx.probe_stream_read(buf, sink), 10, 3, torch)
    flop = dx.probe_mfma_f32(20000, sink)
    ms_m, _ = time_steps(lambda: dx.probe_mfma_f32(20000, sink), 5, 2, torch)
    res = {"stream_read_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "stream_read_bytes": nbytes,
           "mfma_f32_TFLOPs": round(flop / (ms_m * 1e-3) / 1e12, 1)}
    log(f"[bench] probes: stream read {res['stream_read_GBps']:.0f} GB/s over {nbytes / 1e9:.2f} GB, "
        f"fp32 MFMA {res['mfma_f32_TFLOPs']:.1f} TFLOP/s")
    return res


class Legs:
    """Times paths on one resident matrix and records them against their compulsory rows."""

    def __init__(self, n, d, steps, torch, stream_gbs, only=None):
        self.n, self.d, self.steps, self.torch, self.stream_gbs, self.only = n, d, steps, torch, stream_gbs, only
        self.rows = []

    def timed(self, name, fn, rows, warmup=2, **extra):
        if self.only and self.only not in name:
            return None
        ms, _ = time_steps(fn, self.steps, warmup, self.torch)
        gbs = rows * self.d * 4 / (ms * 1e-3) / 1e9
        rec = {"path": name, "ms_per_step": round(ms, 5),
               "GBps_aggregated": round(self.n * self.d * 4 / (ms * 1e-3) / 1e9, 1),
               "rows_moved": rows, "hbm_frac_algorithmic": round(gbs / HBM_PEAK_GBS, 4),
               "frac_of_measured_stream": round(gbs / self.stream_gbs, 4) if self.stream_gbs else None, **extra}
        self.rows.append(rec)
        log(f"[bench] {name}: {ms:.4f} ms/step, {rec['hbm_frac_algorithmic'] * 100:.1f}% of HBM peak over {rows} rows")
        return rec


def mean_estimation_paths(dx, workloads, torch, np, steps, d=100):
    """The synthetic mean-estimation setting of Section 5.3 (220000 nodes in groups of 11, d = 100):
    the DETOX step and the same aggregator over all rows.  A step lasts tens of microseconds, less
    than the host needs to enqueue it, so each path is timed twice: called from Python, and as a
    replayed HIP graph of 20 calls (the GPU's own time; every replay is checked against the eager
    result)."""
    from paper_1907_12205_amd.binding import StepBuffers
    w = workloads.mean_estimation(d)
    n, r, q = w.n, w.r, w.q
    G = torch.from_numpy(w.matrix()).cuda()
    B = w.detox[0]["B"]
    buf = StepBuffers(n, d, r, B, G.device)
    out = torch.empty(d, dtype=torch.float32, device=G.device)
    ws_m = torch.empty(dx.workspace_bytes("coord_median_many", n, d), dtype=torch.uint8, device=G.device)
    ws_g = torch.empty(dx.workspace_bytes("geomedian_many", n, d), dtype=torch.uint8, device=G.device)
    paths = [
        (f"DETOX coord-median, B={B}", lambda: dx.detox_step(G, r, q, B, "coord_median", buffers=buf), buf.out),
        (f"DETOX geometric median, B={B}, 50 iterations", lambda: dx.detox_step(G, r, q, B, "geomedian", buffers=buf), buf.out),
        (f"vanilla coord-median over {n} rows", lambda: dx.robust_coord_median_many(G, out=out, ws=ws_m), out),
        (f"vanilla geometric median over {n} rows, 50 iterations", lambda: dx.robust_geomedian_many(G, 50, 1e-8, out=out, ws=ws_g), out),
    ]
    rep, res = 20, []
    for name, fn, result in paths:
        ms_eager, _ = time_steps(fn, max(steps, 5), 3, torch)
        want = result.clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(rep):
                fn()
        same = True
        for _ in range(3):
            result.zero_()
            graph.replay()
            torch.cuda.synchronize()
            same = same and bool(torch.equal(result, want))
        ms_graph, _ = time_steps(graph.replay, 10, 2, torch)
        ms_graph /= rep
        res.append({"path": name, "ms_per_step_eager": round(ms_eager, 5), "ms_per_step_graph": round(ms_graph, 5),
                    "GBps_aggregated": round(n * d * 4 / (ms_graph * 1e-3) / 1e9, 1),
                    "hbm_frac_algorithmic": round(n * d * 4 / (ms_graph * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "graph_replays_match_eager": same})
        log(f"[bench] mean estimation, {name}: {ms_graph:.4f} ms/step on the GPU ({ms_eager:.4f} called from Python), "
            f"replays match: {same}")
    return {"workload": f"{w.name}: n={n}, r={r}, q={q}, d={d}, {w.attack}", "paths": res}


def device_matrix(torch, n, r, d, byz_rows, kind, seed=20190712):
    """An n x d matrix with the replication structure of the workloads, generated on the device
    (timing only; the seeded host generators of `workloads` serve the parity tests): one base
    vector per node group copied to its members, Byzantine rows overwritten.
      kind "student_t": base 1e-3 * t(3), Byzantine rows uniform in [-1, 1];
      kind "normal"   : base N(0, 1e-3), Byzantine rows constant +-100."""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    G = torch.empty((n, d), dtype=torch.float32, device="cuda:0")
    for j in range(n // r):
        z = torch.randn(d, device="cuda:0", generator=g)
        if kind == "student_t":
            chi = sum(torch.randn(d, device="cuda:0", generator=g) ** 2 for _ in range(3)) / 3.0
            z = z / chi.sqrt()
            z *= 1e-3
        else:
            z *= 1e-3 ** 0.5
        for k in range(r):
            G[j * r + k].copy_(z)
        del z
    for t, i in enumerate(byz_rows):
        if kind == "student_t":
            G[i].uniform_(-1.0, 1.0, generator=g)
        else:
            G[i].fill_(100.0 if t % 2 == 0 else -100.0)
    torch.cuda.synchronize()
    return G


def gram_roofline(n, d, kernel_ms, pr):
    """The Gram kernel of more than 8 rows.  It reads the rows once (4 n d bytes) and does the
    method's n(n+1)/2 fp32 multiply-adds per column as six bf16 matrix instructions per 16x16 tile
    and 32 columns (operands cut into three bf16 pieces): reported against the HBM peak, with the
    rate on the method's own operations beside the fp32 matrix-core peak it no longer depends on,
    and the bf16 operations actually issued (padded tiles included) against the bf16 peak."""
    flop = n * (n + 1) / 2 * 2.0 * d
    tiles = (n + 15) // 16
    issued = 6.0 * (tiles * (tiles + 1) / 2) * 256 * 2.0 * d
    sec = kernel_ms * 1e-3
    gbs = 4.0 * n * d / sec / 1e9
    return {"bound": "hbm", "kernel": "gram_mfma_bf16x3", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4),
            "frac_of_measured_stream": round(gbs / pr["stream_read_GBps"], 4) if pr.get("stream_read_GBps") else None,
            "method_fp32_TFLOPs": round(flop / sec / 1e12, 1),
            "method_fp32_vs_fp32_mfma_peak": round(flop / sec / 1e12 / MFMA_F32_PEAK_TFLOPS, 4),
            "issued_bf16_TFLOPs": round(issued / sec / 1e12, 1),
            "issued_bf16_vs_bf16_mfma_peak": round(issued / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "algorithmic_flop_per_launch": flop, "algorithmic_bytes_per_launch": 4.0 * n * d,
            "kernel_ms": round(kernel_ms, 5), "traffic": None}


def big_workloads(dx, workloads, torch, np, steps, pr, only):
    """The two d = 25,000,000 workloads: DETOX pipelines and vanilla aggregators, device-generated data."""
    from paper_1907_12205_amd.binding import StepBuffers
    res = []
    d = 25_000_000
    # ---- n = 45, r = 3, q = 5, heavy-tailed ------------------------------------------------------
    n, r, q = 45, 3, 5
    byz = workloads.place_byzantine(workloads.DEFAULT_SEED, n, r, q, 1)
    G = device_matrix(torch, n, r, d, byz, "student_t")
    legs = Legs(n, d, steps, torch, pr["stream_read_GBps"], only)
    out = torch.empty(d, dtype=torch.float32, device=G.device)
    b15 = StepBuffers(n, d, r, 15, G.device, materialise=False)
    b5 = StepBuffers(n, d, r, 5, G.device, materialise=False)
    legs.timed("DETOX Bulyan over the 15 votes, f=1", lambda: dx.detox_step(G, r, q, 15, "bulyan", f=1, buffers=b15), n + 13 + 1)
    legs.timed("DETOX coord-median, B=5 (one pass)", lambda: dx.detox_step(G, r, q, 5, "coord_median", buffers=b5), n + 1)
    ws = torch.empty(dx.workspace_bytes("bulyan", n, d), dtype=torch.uint8, device=G.device)
    legs.timed("vanilla Bulyan over 45 rows, f=5", lambda: dx.robust_bulyan(G, 5, out=out, ws=ws), n + 35 + 1)
    res.append({"workload": f"cfg4 shape: n={n}, r={r}, q={q}, d={d}, Student-t(3) base, uniform Byzantine rows; "
                            "generated on the device", "paths": legs.rows})
    del G, b15, b5, ws, out
    torch.cuda.empty_cache()
    # ---- n = 105, r = 5, q = 10 ------------------------------------------------------------------
    n, r, q = 105, 5, 10
    byz = workloads.place_byzantine(workloads.DEFAULT_SEED, n, r, q, 2)
    G = device_matrix(torch, n, r, d, byz, "normal")
    legs = Legs(n, d, max(steps // 2, 3), torch, pr["stream_read_GBps"], only)
    out = torch.empty(d, dtype=torch.float32, device=G.device)
    b7 = StepBuffers(n, d, r, 7, G.device, materialise=False)
    b21 = StepBuffers(n, d, r, 21, G.device, materialise=False)
    legs.timed("DETOX geometric median, B=7, 50 iterations", lambda: dx.detox_step(G, r, q, 7, "geomedian", buffers=b7), n + 7 + 7 + 1)
    legs.timed("DETOX Bulyan over the 21 votes, f=2", lambda: dx.detox_step(G, r, q, 21, "bulyan", f=2, buffers=b21), n + 17 + 1)
    legs.timed("vanilla coord-median over 105 rows", lambda: dx.robust_coord_median(G, out=out), n + 1)
    ws = torch.empty(dx.workspace_bytes("multikrum", n, d), dtype=torch.uint8, device=G.device)
    fn = lambda: dx.robust_multikrum(G, 10, 95, out=out, ws=ws, with_scores=False)
    rec = legs.timed("vanilla Multi-Krum over 105 rows, f=10, m=95", fn, n + 95 + 1)
    if rec is not None:
        km = traced_kernels(dx, fn, 3, np)
        rec["kernel_ms"] = {k: round(v, 5) for k, v in km.items()}
        if "gram_mfma_bf16x3" in km:
            rec["roofline"] = gram_roofline(n, d, km["gram_mfma_bf16x3"], pr)
            log(f"[bench] Gram kernel of 105 rows: {km['gram_mfma_bf16x3']:.3f} ms = {rec['roofline']['achieved']:.0f} GB/s "
                f"({rec['roofline']['frac'] * 100:.1f}% of HBM peak), {rec['roofline']['method_fp32_TFLOPs']:.1f} TFLOP/s on the "
                f"method's fp32 operations ({rec['roofline']['method_fp32_vs_fp32_mfma_peak'] * 100:.0f}% of the fp32 MFMA peak)")
    res.append({"workload": f"cfg5 shape: n={n}, r={r}, q={q}, d={d}, N(0,1e-3) base, constant +-100 Byzantine rows; "
                            "generated on the device", "paths": legs.rows})
    del G
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload index 1..5 (3 = headline)")
    ap.add_argument("--d", type=int, default=None, help="override the dimension (debugging)")
    ap.add_argument("--ld", type=int, default=None, help="row stride in elements (default: d rounded up to 64)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-vanilla", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other aggregators' timings")
    ap.add_argument("--no-mean-estimation", action="store_true", help="skip the many-short-rows setting")
    ap.add_argument("--no-big", action="store_true", help="skip the two d = 25,000,000 workloads")
    ap.add_argument("--only", default=None, help="time only the paths whose name contains this (profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the parameter-server step on ONE GPU (the step has no "
                 "inter-GPU part); run with --gpus 1")

    import numpy as np
    import torch

    import paper_1907_12205_amd as dx
    import workloads
    from paper_1907_12205_amd.binding import StepBuffers

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    dx.lib()   # fails loudly if the HIP library has not been built

    t0 = time.time()
    w = workloads.config(args.config, d=args.d)
    n, r, q, d = w.n, w.r, w.q, w.d
    ld = args.ld or (d + 63) // 64 * 64            # rows padded to 256 bytes: 16-byte loads everywhere
    G = w.to_device("cuda:0", ld=ld)
    spec = w.detox[0]
    B, agg = spec["B"], spec["aggregator"]
    groups = n // r
    log(f"[bench] workload {w.name}: n={n} r={r} q={q} d={d} ld={ld} attack={w.attack} "
        f"({n * d * 4 / 1e9:.3f} GB resident, generated in {time.time() - t0:.1f}s)")
    pr = probes(dx, torch, G)

    # the block means are not written to memory (Zhat = NULL): the fast mode of detox_step
    buf = StepBuffers(n, d, r, B, G.device, materialise=False)
    kw = dict(f=spec.get("f", -1), m=spec.get("m", -1), iters=spec.get("iters", 50), eps=spec.get("eps", 1e-8))

    def detox_step():
        dx.detox_step(G, r, q, B, agg, buffers=buf, **kw)

    ms_step, wall_ms = time_steps(detox_step, args.steps, args.warmup, torch)
    in_bytes = n * d * 4
    value = in_bytes / (ms_step * 1e-3) / 1e9
    log(f"[bench] DETOX step ({agg}, B={B}): {ms_step:.4f} ms/step (host wall {wall_ms:.4f}), "
        f"{value:.1f} GB/s of gradients aggregated")

    # ---- dominant kernel, timed by the library's own HIP events on the launch stream --------
    kernel_ms = traced_kernels(dx, detox_step, args.steps, np)
    dominant = max(kernel_ms, key=kernel_ms.get)
    # algorithmic rows per launch: the one-pass filter kernels read every row of G once; the
    # median variant also writes the d-vector
    alg_rows = {"filter_block_mean_gram": n, "filter_block_mean_median": n + 1, "filter": n,
                "filter_block_mean": n + B, "filter_votes_gram": n}
    alg_bytes = alg_rows.get(dominant, n) * d * 4
    achieved = alg_bytes / (kernel_ms[dominant] * 1e-3) / 1e9
    log("[bench] per-kernel ms: " + ", ".join(f"{k}={v:.4f}" for k, v in kernel_ms.items()))
    traffic, traffic_commit = measured_traffic(agg, n, d)
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_measured_at_commit": traffic_commit,
                "frac_of_measured_stream": round(achieved / pr["stream_read_GBps"], 4),
                "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": round(kernel_ms[dominant], 5)}
    # compulsory traffic of the whole step: n rows in, B block means, m of them out again, 1 result
    step_rows = {"multikrum": n + B + spec.get("m", 0) + 1, "coord_median": n + 1, "trimmed_mean": n + 1,
                 "geomedian": n + B + B + 1, "bulyan": n + (B - 2 * spec.get("f", 0)) + 1}[agg]
    step_alg_bytes = step_rows * d * 4

    legs = Legs(n, d, max(args.steps // 2, 3), torch, pr["stream_read_GBps"], args.only)
    out_o = torch.empty(d, dtype=torch.float32, device=G.device)

    # ---- vanilla comparison: every aggregator the workload names, over all n rows -----------------
    vanilla = []
    if w.vanilla and not args.no_vanilla:
        for v in w.vanilla:
            if v["aggregator"] == "multikrum":
                ws_v = torch.empty(dx.workspace_bytes("multikrum", n, d), dtype=torch.uint8, device=G.device)
                fn = lambda: dx.robust_multikrum(G, v["f"], v["m"], out=out_o, ws=ws_v, with_scores=False)
                rows = n + v["m"] + 1
            elif v["aggregator"] == "bulyan":
                ws_v = torch.empty(dx.workspace_bytes("bulyan", n, d), dtype=torch.uint8, device=G.device)
                fn = lambda: dx.robust_bulyan(G, v["f"], out=out_o, ws=ws_v)
                rows = n + (n - 2 * v["f"]) + 1
            else:
                fn = lambda: dx.robust_coord_median(G, out=out_o)
                rows = n + 1
            ms_v, _ = time_steps(fn, args.steps, args.warmup, torch)
            vk = traced_kernels(dx, fn, min(args.steps, 5), np)
            rec = {"aggregator": v["aggregator"], **{k: v[k] for k in ("f", "m") if k in v},
                   "ms_per_step": round(ms_v, 5), "GBps_aggregated": round(in_bytes / (ms_v * 1e-3) / 1e9, 1),
                   "rows_moved": rows,
                   "hbm_frac_algorithmic": round(rows * d * 4 / (ms_v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                   "frac_of_measured_stream": round(rows * d * 4 / (ms_v * 1e-3) / 1e9 / pr["stream_read_GBps"], 4),
                   "kernel_ms": {k: round(x, 5) for k, x in vk.items()},
                   "detox_speedup": round(ms_v / ms_step, 3)}
            if "gram_mfma_bf16x3" in vk:
                rec["gram_roofline"] = gram_roofline(n, d, vk["gram_mfma_bf16x3"], pr)
            vanilla.append(rec)
            log(f"[bench] vanilla {v['aggregator']}: {ms_v:.4f} ms/step ({rec['hbm_frac_algorithmic'] * 100:.1f}% of HBM peak "
                f"over {rows} rows); DETOX is {ms_v / ms_step:.2f}x faster")

    # ---- the other rows of the hot path on the same resident matrix (reported, not the value) --
    if not args.no_others:
        timed = legs.timed
        timed("filter only (votes)", lambda: dx.detox_majority_filter(G, r), n)
        for other in w.detox[1:]:
            bo = StepBuffers(n, d, r, other["B"], G.device, materialise=False)
            okw = dict(f=other.get("f", -1), m=other.get("m", -1), iters=other.get("iters", 50), eps=other.get("eps", 1e-8))
            rows_o = {"coord_median": n + 1, "bulyan": n + other["B"] - 2 * other.get("f", 0) + 1}.get(other["aggregator"], n + 1)
            timed(f"DETOX {other['aggregator']}, B={other['B']}", lambda: dx.detox_step(G, r, q, other["B"], other["aggregator"], buffers=bo, **okw), rows_o)
        if groups >= 5:
            bm = StepBuffers(n, d, r, 5, G.device, materialise=False)
            timed("DETOX coord-median, B=5 (one pass)", lambda: dx.detox_step(G, r, q, 5, "coord_median", buffers=bm), n + 1)
            timed("DETOX trimmed mean (alpha=1/4), B=5 (one pass)", lambda: dx.detox_step(G, r, q, 5, "trimmed_mean", buffers=bm), n + 1)
            timed("DETOX geometric median, B=5, 50 iterations", lambda: dx.detox_step(G, r, q, 5, "geomedian", buffers=bm), n + 5 + 5 + 1)
        if groups >= 7:
            bb = StepBuffers(n, d, r, groups, G.device, materialise=False)
            timed(f"DETOX Bulyan over the {groups} votes, f=1", lambda: dx.detox_step(G, r, q, groups, "bulyan", f=1, buffers=bb),
                  n + (groups - 2) + 1)
        if groups >= 14:
            # the hierarchy the paper deployed (Section 5.2): robust aggregator inside vote groups, mean across
            ws_h = torch.empty(max(dx.robust_blocks_workspace_bytes(n, d, r, 1), dx.robust_blocks_workspace_bytes(n, d, r, 2)),
                               dtype=torch.uint8, device=G.device)
            timed(f"DETOX A0=Multi-Krum(f=2,m=3) on {groups // 2}+{groups - groups // 2} votes, A1=mean",
                  lambda: dx.detox_step_robust_blocks(G, r, 2, "multikrum", 2, 3, out=out_o, ws=ws_h), n + 2 * 3 + 2 + 1)
            timed(f"DETOX A0=Bulyan(f=2) on all {groups} votes",
                  lambda: dx.detox_step_robust_blocks(G, r, 1, "bulyan", 2, out=out_o, ws=ws_h), n + (groups - 4) + 1)
        timed(f"vanilla coord-median over {n} rows", lambda: dx.robust_coord_median(G, out=out_o), n + 1)
        timed(f"vanilla trimmed mean over {n} rows, {n // 4} off each end",
              lambda: dx.robust_trimmed_mean(G, n // 4, out=out_o), n + 1)
        fb = min(q, (n - 3) // 4)
        ws_b = torch.empty(dx.workspace_bytes("bulyan", n, d), dtype=torch.uint8, device=G.device)
        timed(f"vanilla Bulyan over {n} rows, f={fb}", lambda: dx.robust_bulyan(G, fb, out=out_o, ws=ws_b), n + (n - 2 * fb) + 1)
        if ld != d:
            # the same step on unpadded rows (ld = d): rows off the 16-byte grid when d is not a multiple of 4
            Gu = w.to_device("cuda:0")
            bu = StepBuffers(n, d, r, B, G.device, materialise=False)
            timed(f"DETOX {agg}, B={B}, rows not padded (ld = d = {d})", lambda: dx.detox_step(Gu, r, q, B, agg, buffers=bu, **kw), step_rows)
            del Gu
        if groups >= 5:
            # signSGD pairing: one sign bit per coordinate, two levels of coordinate-wise majority vote
            Sh = workloads.pack_signs(w.matrix(), pad_words=4)       # rows 16-byte aligned: 16-byte loads in the filter
            Sbuf = torch.zeros((n, Sh.strides[0] // 4), dtype=torch.int32, device=G.device)
            S = Sbuf[:, : Sh.shape[1]]
            S.copy_(torch.from_numpy(np.ascontiguousarray(Sh).view(np.int32)))
            ws_s = torch.empty(dx.workspace_bytes("filter", groups, S.shape[1]), dtype=torch.uint8, device=G.device)
            out_s = torch.empty((2, S.shape[1]), dtype=torch.int32, device=G.device)
            timed("DETOX + signSGD majority vote, bit-packed signs, B=5",
                  lambda: dx.detox_sign_majority(S, d, r, 5, ws=ws_s, out=out_s), (n + 2) / 32)
            del S, Sbuf

    mean_est = None
    if not args.no_others and not args.no_mean_estimation and not args.only:
        mean_est = mean_estimation_paths(dx, workloads, torch, np, args.steps)

    # ---- CPU oracle on the host cores (a reported baseline, not the target) ------------------
    cpu = None
    if not args.no_cpu:
        import oracle

        Gh = w.matrix()
        okw = {k: v for k, v in spec.items() if k not in ("B", "aggregator")}
        ref_out, ref_w, _ = oracle.detox_step(Gh, r, B, agg, **okw)      # untimed: pages in, threads up
        reps, t1 = 0, time.perf_counter()
        while reps < 50 and (reps < 3 or time.perf_counter() - t1 < 10.0):
            ref_out, ref_w, _ = oracle.detox_step(Gh, r, B, agg, **okw)
            reps += 1
        t_cpu = (time.perf_counter() - t1) / reps
        got = buf.out.cpu().numpy().astype(np.float64)
        err = float(np.linalg.norm(got - ref_out) / max(np.linalg.norm(ref_out), 1e-300))
        same_w = buf.winner.cpu().numpy().tolist() == ref_w.tolist()
        cpu = {"value": round(in_bytes / t_cpu / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"the full workload ({n} x {d}), mean of {reps} repetitions of the DETOX step",
               "ms_per_step": round(t_cpu * 1e3, 2), "gpu_matches_oracle": bool(same_w and err <= 1e-5),
               "rel_l2_vs_oracle": err}
        log(f"[bench] CPU oracle: {t_cpu * 1e3:.1f} ms on {cpu['cores']} threads; GPU rel-L2 vs oracle {err:.2e}, "
            f"votes equal: {same_w}")
        if vanilla and w.vanilla[0]["aggregator"] == "multikrum" and n * d <= 6e8:
            t1 = time.perf_counter()
            oracle.multikrum(Gh, w.vanilla[0]["f"], w.vanilla[0]["m"])
            cpu["vanilla_ms_per_step"] = round((time.perf_counter() - t1) * 1e3, 1)
        del Gh

    big = None
    if not args.no_big and args.config == 3 and args.d is None:
        del G, buf
        torch.cuda.empty_cache()
        big = big_workloads(dx, workloads, torch, np, max(args.steps // 2, 3), pr, args.only)

    line = {
        "metric": "aggregated gradient GB/s and ms/step (DETOX vs vanilla), % HBM roofline",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: n={n}, r={r}, q={q}, d={d}, {w.attack}; filter -> {n // r} votes -> "
                               f"{B} block means -> {agg}", "ld": ld, **{k: v for k, v in spec.items() if k != "aggregator"}},
        "step_rows_moved": step_rows,
        "step_hbm_frac_algorithmic": round(step_alg_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "step_frac_of_measured_stream": round(step_alg_bytes / (ms_step * 1e-3) / 1e9 / pr["stream_read_GBps"], 4),
        "kernel_ms": {k: round(v, 5) for k, v in kernel_ms.items()},
        "roofline": roofline, "measured_ceilings": pr, "vanilla": vanilla, "other_paths": legs.rows,
        "other_workloads": big, "mean_estimation": mean_est, "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
