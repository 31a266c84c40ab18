#!/usr/bin/env python3
"""Benchmark of the DETOX parameter-server step on one MI355X.

Workload (the one the headline metric is quoted on): n = 45 nodes, r = 3, q = 5 Byzantine
(ALIE attack), d = 11,173,962 fp32 (ResNet-18-sized), synthetic and seeded.  One "step" is one
pass of the whole hot path over the resident n x d matrix:
    majority-vote filter -> 15 votes -> 5 block means -> Multi-Krum(f=1, m=3) -> d-vector.
The same run also times the vanilla comparison (Multi-Krum over all 45 rows, f=5, m=40), the
dominant kernel on its own (per-kernel HIP events inside the library) and the CPU oracle on the
host cores.  Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak


def measured_traffic(agg, n, d):
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE for this workload (the committed summary under profiles/), or None."""
    import re
    path = os.path.join(ROOT, "profiles", f"detox_step_{agg}__n{n}_d{d}.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\[.*\]: (\d+)", open(path).read(), re.M)
        return int(m.group(1)) if m else None
    except OSError:
        return None


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload index 1..5 (3 = headline)")
    ap.add_argument("--d", type=int, default=None, help="override the dimension (debugging)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-vanilla", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other aggregators' timings")
    ap.add_argument("--no-mean-estimation", action="store_true", help="skip the many-short-rows setting")
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
    ld = (d + 63) // 64 * 64                       # rows padded to 256 bytes: 16-byte loads everywhere
    G = w.to_device("cuda:0", ld=ld)
    spec = w.detox[0]
    B, agg = spec["B"], spec["aggregator"]
    log(f"[bench] workload {w.name}: n={n} r={r} q={q} d={d} ld={ld} attack={w.attack} "
        f"({n * d * 4 / 1e9:.3f} GB resident, generated in {time.time() - t0:.1f}s)")

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
    with dx.trace() as tr:
        for _ in range(args.steps):
            detox_step()
        recs = tr.records()
    per_kernel = {}
    for name, ms in recs:
        per_kernel.setdefault(name, []).append(ms)
    kernel_ms = {k: float(np.mean(v)) for k, v in per_kernel.items()}
    dominant = max(kernel_ms, key=kernel_ms.get)
    # algorithmic rows per launch: the one-pass filter kernels read every row of G once; the
    # median variant also writes the d-vector
    alg_rows = {"filter_block_mean_gram": n, "filter_block_mean_median": n + 1, "filter": n,
                "filter_block_mean": n + B}
    alg_bytes = alg_rows.get(dominant, n) * d * 4
    achieved = alg_bytes / (kernel_ms[dominant] * 1e-3) / 1e9
    log("[bench] per-kernel ms: " + ", ".join(f"{k}={v:.4f}" for k, v in kernel_ms.items()))
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(agg, n, d),
                "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": round(kernel_ms[dominant], 5)}
    # compulsory traffic of the whole step: n rows in, B block means, m of them out again, 1 result
    step_alg_bytes = (n + B + spec.get("m", 0) + 1) * d * 4 if agg == "multikrum" else None

    # ---- vanilla comparison: the same aggregator over all n rows ------------------------------
    vanilla = None
    if w.vanilla and not args.no_vanilla:
        v = w.vanilla[0]
        out_v = torch.empty(d, dtype=torch.float32, device=G.device)
        if v["aggregator"] == "multikrum":
            ws_v = torch.empty(dx.workspace_bytes("multikrum", n, d), dtype=torch.uint8, device=G.device)
            fn = lambda: dx.robust_multikrum(G, v["f"], v["m"], out=out_v, ws=ws_v, with_scores=False)
            rows = n + v["m"] + 1
        elif v["aggregator"] == "bulyan":
            ws_v = torch.empty(dx.workspace_bytes("bulyan", n, d), dtype=torch.uint8, device=G.device)
            fn = lambda: dx.robust_bulyan(G, v["f"], out=out_v, ws=ws_v)
            rows = n + (n - 2 * v["f"]) + 1
        else:
            fn = lambda: dx.robust_coord_median(G, out=out_v)
            rows = n + 1
        ms_v, _ = time_steps(fn, args.steps, args.warmup, torch)
        with dx.trace() as tr:
            for _ in range(min(args.steps, 5)):
                fn()
            recs = tr.records()
        vk = {}
        for name, ms in recs:
            vk.setdefault(name, []).append(ms)
        vanilla = {"aggregator": v["aggregator"], **{k: v[k] for k in ("f", "m") if k in v},
                   "ms_per_step": round(ms_v, 5), "GBps_aggregated": round(in_bytes / (ms_v * 1e-3) / 1e9, 1),
                   "hbm_frac_algorithmic": round(rows * d * 4 / (ms_v * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                   "kernel_ms": {k: round(float(np.mean(x)), 5) for k, x in vk.items()},
                   "detox_speedup": round(ms_v / ms_step, 3)}
        log(f"[bench] vanilla {v['aggregator']}: {ms_v:.4f} ms/step; DETOX is {ms_v / ms_step:.2f}x faster")

    # ---- the other rows of the hot path on the same resident matrix (reported, not the value) --
    others = []
    if not args.no_others:
        def timed(name, fn, rows):
            ms, _ = time_steps(fn, max(args.steps // 2, 3), 2, torch)
            others.append({"path": name, "ms_per_step": round(ms, 5),
                           "GBps_aggregated": round(in_bytes / (ms * 1e-3) / 1e9, 1),
                           "hbm_frac_algorithmic": round(rows * d * 4 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
        groups = n // r
        out_o = torch.empty(d, dtype=torch.float32, device=G.device)
        timed("filter only (votes)", lambda: dx.detox_majority_filter(G, r), n)
        if groups >= 5:
            bm = StepBuffers(n, d, r, 5, G.device, materialise=False)
            timed("DETOX coord-median, B=5 (one pass)", lambda: dx.detox_step(G, r, q, 5, "coord_median", buffers=bm), n + 1)
            timed("DETOX trimmed mean (alpha=1/4), B=5 (one pass)", lambda: dx.detox_step(G, r, q, 5, "trimmed_mean", buffers=bm), n + 1)
            timed("DETOX geometric median, B=5, 50 iterations", lambda: dx.detox_step(G, r, q, 5, "geomedian", buffers=bm), n + groups + 1)
        if groups >= 7:
            bb = StepBuffers(n, d, r, groups, G.device, materialise=False)
            # 9..16 votes: their Gram matrix comes out of the filter pass, so the votes are read once more
            # only for the trimming (more votes: also once for the Gram matrix)
            timed(f"DETOX Bulyan over the {groups} votes, f=1", lambda: dx.detox_step(G, r, q, groups, "bulyan", f=1, buffers=bb),
                  n + (0 if 8 < groups <= 16 else groups) + (groups - 2) + 1)
        if groups >= 14:
            # the hierarchy the paper deployed (Section 5.2): robust aggregator inside vote groups, mean across
            gram_rows = 0 if 8 < groups <= 16 else groups   # 9..16 votes: their Gram matrix comes with the filter pass
            ws_h = torch.empty(max(dx.robust_blocks_workspace_bytes(n, d, r, 1), dx.robust_blocks_workspace_bytes(n, d, r, 2)),
                               dtype=torch.uint8, device=G.device)
            timed(f"DETOX A0=Multi-Krum(f=2,m=3) on {groups // 2}+{groups - groups // 2} votes, A1=mean",
                  lambda: dx.detox_step_robust_blocks(G, r, 2, "multikrum", 2, 3, out=out_o, ws=ws_h), n + gram_rows + 2 * 3 + 2 + 2 + 1)
            timed(f"DETOX A0=Bulyan(f=2) on all {groups} votes",
                  lambda: dx.detox_step_robust_blocks(G, r, 1, "bulyan", 2, out=out_o, ws=ws_h), n + gram_rows + (groups - 4) + 1)
        timed(f"vanilla coord-median over {n} rows", lambda: dx.robust_coord_median(G, out=out_o), n + 1)
        timed(f"vanilla trimmed mean over {n} rows, {n // 4} off each end",
              lambda: dx.robust_trimmed_mean(G, n // 4, out=out_o), n + 1)
        fb = min(q, (n - 3) // 4)
        ws_b = torch.empty(dx.workspace_bytes("bulyan", n, d), dtype=torch.uint8, device=G.device)
        timed(f"vanilla Bulyan over {n} rows, f={fb}", lambda: dx.robust_bulyan(G, fb, out=out_o, ws=ws_b), n + (n - 2 * fb) + 1)
        if groups >= 5:
            # signSGD pairing: one sign bit per coordinate, two levels of coordinate-wise majority vote
            S = torch.from_numpy(workloads.pack_signs(w.matrix()).view(np.int32)).to(G.device)
            ws_s = torch.empty(dx.workspace_bytes("filter", groups, S.shape[1]), dtype=torch.uint8, device=G.device)
            out_s = torch.empty((2, S.shape[1]), dtype=torch.int32, device=G.device)
            timed("DETOX + signSGD majority vote, bit-packed signs, B=5",
                  lambda: dx.detox_sign_majority(S, d, r, 5, ws=ws_s, out=out_s), (n + groups + 2) / 32)
        for o in others:
            log(f"[bench] {o['path']}: {o['ms_per_step']:.4f} ms/step, {o['hbm_frac_algorithmic'] * 100:.1f}% of HBM peak (algorithmic bytes)")

    mean_est = None
    if not args.no_others and not args.no_mean_estimation:
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

    line = {
        "metric": "aggregated gradient GB/s and ms/step (DETOX vs vanilla), % HBM roofline",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: n={n}, r={r}, q={q}, d={d}, {w.attack}; filter -> {n // r} votes -> "
                               f"{B} block means -> {agg}", "ld": ld, **{k: v for k, v in spec.items() if k != "aggregator"}},
        "step_hbm_frac_algorithmic": (round(step_alg_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                      if step_alg_bytes else None),
        "kernel_ms": {k: round(v, 5) for k, v in kernel_ms.items()},
        "roofline": roofline, "vanilla": vanilla, "other_paths": others, "mean_estimation": mean_est,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
