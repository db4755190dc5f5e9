#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: Nystrom factor G = K(X, L) W^T followed by the margin sweep G w.

One "step" is one pass of the whole path over the workload: squared norms, kernel block panels
(distance contraction with fused exp), whitening product, then the sweep over all rows of G.
Inputs (X, L, W, w) are resident in HBM before the timed region; the one-off host preparation of W
(landmark kernel matrix + eigendecomposition) is timed separately and reported, not counted.

Prints ONE JSON line.  `value` is rows per second through the whole path (factor + sweep).
`roofline` describes the dominant kernel (the whitening product) from HIP events recorded on the
launch stream around every launch inside the timed steps; `roofline_sweep` does the same for the
margin sweep against HBM bandwidth; `cpu_baseline` is the double-precision oracle timed on the host
cores on a bounded row sample of the same workload.
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

FP32_MFMA_PEAK_TFLOPS = 157.3   # 256 CU x 256 FLOP/clk x 2.4 GHz
HBM_PEAK_GBPS = 8000.0



def measured_traffic(workload, panel_rows):
    """HBM-side bytes per launch of the dominant kernel and of the sweep, as the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE runs recorded them in profiles/factor_and_sweep_<workload>_hbm_traffic.txt (the line starting with
    '#@').  (None, None) when there is no such record or it was taken with another panel size."""
    path = os.path.join(ROOT, "profiles", f"factor_and_sweep_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("#@"):
                kv = dict(item.split("=", 1) for item in line[2:].split())
                if int(kv.get("panel_rows", -1)) != int(panel_rows):
                    return None, None
                return float(kv["dominant_bytes_per_launch"]), float(kv["sweep_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None, None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=None, choices=["tiny", "small", "digit", "cnn", "highrank"],
                    help="default: highrank for the factor path (the largest configuration that fits one GPU), "
                         "cnn for predict and whiten, digit for stream and sparse")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tile", default="auto", choices=["auto", "128x128", "256x128", "256x256", "64x128"])
    ap.add_argument("--workspace-mult", type=float, default=1.0)
    ap.add_argument("--panel-rows", type=int, default=0,
                    help="factor: size the workspace for kernel-block panels of this many rows (a multiple of 256; "
                         "0 = the library's recommendation)")
    ap.add_argument("--path", default="factor", choices=["factor", "solver", "predict", "stream", "whiten", "sparse",
                                                         "multi", "calibrate"],
                    help="factor: Nystrom factor + margin sweep (default); solver: batched dual coordinate ascent "
                         "on G; predict: scores of new points; stream: the factor copied to pinned host memory as it is made; whiten: the one-off preparation "
                         "(steps 1a-1c) on the device; sparse: the factor from X in compressed-row form; multi: one pass over G "
                         "against --vectors weight vectors; calibrate: a "
                         "plain 1 GiB device-to-device copy, the known traffic the FETCH_SIZE / WRITE_SIZE counters "
                         "are scaled by")
    ap.add_argument("--classifiers", type=int, default=10, help="predict: number of classifiers scored at once")
    ap.add_argument("--vectors", type=int, default=32, help="multi: weight vectors swept at once")
    ap.add_argument("--whiten", default="device", choices=["device", "host"],
                    help="steps 1a-1c (one-off preparation, outside the timed region): lpd_whiten on the GPU, or the "
                         "host routine")
    ap.add_argument("--density", type=float, default=None,
                    help="sparse: share of non-zeros of the digit-shaped recipe (default: its own 0.2)")
    ap.add_argument("--csr-route", default="auto", choices=["auto", "dense", "gather"],
                    help="sparse: route of the compressed-row entry points (auto = by density)")
    ap.add_argument("--chunk-rows", type=int, default=0, help="stream: rows per chunk (0 = the library's suggestion)")
    ap.add_argument("--random-w", action="store_true",
                    help="skip the host eigendecomposition and use a random W (tuning only; marks the line invalid)")
    args = ap.parse_args()
    if args.workload is None:
        args.workload = {"factor": "highrank", "predict": "cnn", "whiten": "cnn", "stream": "digit", "sparse": "digit",
                         "solver": "small", "calibrate": "tiny"}[args.path]
    return args


def whiten(args, lpd, L, gamma):
    """W on the host (float32 CPU tensor) and the rank, by the routine --whiten names."""
    import torch
    if args.whiten == "host":
        W, eig, rank = lpd.lpd_whiten_host(L.cpu(), gamma)
        return W, rank
    W, eig, rank = lpd.lpd_whiten(L, gamma)
    W = W.cpu()
    torch.cuda.empty_cache()        # the eigensolver scratch (2 B^2 doubles) goes back to the pool
    return W, rank


def cpu_baseline(orc, wl, Xs, L, W, w, target_s):
    """Oracle (factor rows + margins over them) on a row sample sized for about `target_s` seconds."""
    import numpy as np
    probe = min(32, Xs.shape[0])
    t0 = time.perf_counter()
    orc.nystrom_factor(Xs[:probe], L, wl.gamma, W)
    per_row = (time.perf_counter() - t0) / probe
    m = int(max(probe, min(Xs.shape[0], target_s / max(per_row, 1e-9))))
    t0 = time.perf_counter()
    G = orc.nystrom_factor(Xs[:m], L, wl.gamma, W)
    t_factor = time.perf_counter() - t0
    G32 = G.astype(np.float32)
    t0 = time.perf_counter()
    orc.margins(G32, w)
    t_sweep = time.perf_counter() - t0
    flop_row = 2.0 * wl.B * (wl.d + W.shape[0])
    return {
        "value": m / (t_factor + t_sweep), "unit": "rows/s", "cores": orc.num_threads(), "kind": "oracle",
        "sample": f"first {m} of {wl.n} rows of the '{wl.name}' workload (all {wl.B} landmarks, full W); "
                  f"factor {t_factor:.2f} s + sweep {t_sweep:.4f} s in double precision",
        "factor_gflops": m * flop_row / t_factor / 1e9,
        "sweep_gbps": 4.0 * m * W.shape[0] / max(t_sweep, 1e-9) / 1e9,
    }


def solver_problems(wl, comp, folds=5, Cs=(0.25, 1.0, 4.0, 16.0, 64.0)):
    """One-versus-one pairs of the 10 mixture components x C grid x folds (training part of each fold)."""
    import numpy as np
    rng = np.random.default_rng(wl.seed(3))
    fold_of = rng.integers(0, folds, size=wl.n)
    probs = []
    for c0 in range(10):
        for c1 in range(c0 + 1, 10):
            pair = np.nonzero((comp == c0) | (comp == c1))[0]
            for f in range(folds):
                rows = pair[fold_of[pair] != f]
                rows = rows[rng.permutation(len(rows))].astype(np.int64)      # randomised visiting order
                yy = np.where(comp[rows] == c0, 1.0, -1.0).astype(np.float32)
                for C in Cs:
                    probs.append((rows, yy, C))
    return probs


def bench_solver(args):
    """Stage 2 on the GPU: all binary problems of a one-vs-one x C-grid x 5-fold run on the 'small' workload."""
    import numpy as np
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS["small"]
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    W_host, rank = whiten(args, lpd, L, wl.gamma)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, W_host.to(dev), G, lpd.alloc_workspace(wl.n, wl.d, wl.B, dev), r=rank)
    gsq = lpd.lpd_row_sqnorms(G, r=rank)
    comp = workloads.mixture_components(wl).numpy()
    probs = solver_problems(wl, comp)
    P = len(probs)
    off = np.zeros(P + 1, dtype=np.int64)
    for i, pr in enumerate(probs):
        off[i + 1] = off[i] + len(pr[0])
    rows = torch.from_numpy(np.concatenate([pr[0] for pr in probs])).to(dev)
    y = torch.from_numpy(np.concatenate([pr[1] for pr in probs])).to(dev)
    C = torch.tensor([pr[2] for pr in probs], dtype=torch.float32, device=dev)
    off_d = torch.from_numpy(off).to(dev)
    alpha = torch.zeros(int(off[-1]), dtype=torch.float32, device=dev)
    w = torch.empty((P, rank), dtype=torch.float32, device=dev)
    ws = torch.empty(lpd.lpd_cd_solve_workspace(P, int(off[-1])), dtype=torch.uint8, device=dev)
    eps, max_epochs = 1e-3, 10000

    def step():
        alpha.zero_()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        _, _, st = lpd.lpd_cd_solve(G, gsq, off_d, rows, y, C, alpha, w, eps=eps, max_epochs=max_epochs, r=rank,
                                    workspace=ws, validate=False)   # reading the status back synchronises
        e1.record()
        torch.cuda.synchronize()
        return st, e0.elapsed_time(e1)

    for _ in range(args.warmup):
        step()
    t0 = time.perf_counter()
    recs = [step() for _ in range(args.steps)]
    elapsed = time.perf_counter() - t0
    st = recs[-1][0]
    steps_per_solve = int(st["steps"].sum())
    ms_kernel = sum(ms for _, ms in recs) / len(recs)
    bytes_per_launch = 4.0 * rank * steps_per_solve
    gbps = bytes_per_launch / (ms_kernel * 1e-3) / 1e9
    out = {
        "metric": "dual_coordinate_ascent_steps_per_s", "value": steps_per_solve * len(recs) / elapsed,
        "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / len(recs), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "small: one-vs-one (45 pairs) x 5 C values x 5 folds", "n": wl.n, "B": wl.B,
                   "rank": rank, "problems": P, "rows_per_problem": float(np.mean(np.diff(off))),
                   "eps": eps, "shrink_k": 5, "eta": 0.05},
        "solve": {"problems_per_s": P * len(recs) / elapsed, "ms_per_problem": elapsed * 1e3 / len(recs) / P,
                  "cd_steps_per_solve": steps_per_solve, "converged": int(st["converged"].sum()),
                  "mean_epochs": float(st["epochs"].mean()), "mean_final_active": float(st["active"].mean()),
                  # the kernel ends with its longest problem: its step count prices the dependent chain
                  "max_steps_one_problem": int(st["steps"].max()), "mean_steps_one_problem": float(st["steps"].mean()),
                  "ns_per_step_longest_problem": ms_kernel * 1e6 / max(int(st["steps"].max()), 1)},
        "roofline": {"kernel": "cd_solve_kernel", "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "bytes_per_launch": bytes_per_launch,
                     "avg_launch_ms": ms_kernel,
                     # profiles/cd_solve_small_ovo_kernel_stats.txt: FETCH_SIZE 3.7741e8 KiB x 2.0 + WRITE_SIZE 2.4194e6 KiB
                     "traffic": 3.7741e8 * 1024 * 2.0 + 2.4194e6 * 1024,
                     "note": "4*r bytes of G per coordinate step; each row read misses L2 (a problem cycles through "
                             "65 MB of rows); the kernel ends with its longest problem, one dependent step after the other"},
    }
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import lpd_oracle as orc
        Gh = G.cpu().numpy()
        cores = os.cpu_count() or 1
        sample = probs[:: max(1, P // (2 * cores))][: 2 * cores]
        orc.set_num_threads(1)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as ex:
            res = list(ex.map(lambda pr: orc.cd_solve(Gh, pr[0], pr[1], pr[2], eps=eps, max_epochs=max_epochs,
                                                      r=rank)[2], sample))
        t_cpu = time.perf_counter() - t0
        cpu_steps = sum(r_["steps"] for r_ in res)
        out["cpu_baseline"] = {"value": cpu_steps / t_cpu, "unit": "steps/s", "cores": cores, "kind": "oracle",
                               "sample": f"{len(sample)} of the {P} problems, one per thread, double precision, "
                                         f"{t_cpu:.1f} s", "problems_per_s": len(sample) / t_cpu,
                               "gpu_over_cpu": out["value"] / (cpu_steps / t_cpu)}
    print(json.dumps(out))


def bench_predict(args):
    """Prediction: scores of c classifiers for the first rows of the workload taken as new points."""
    import numpy as np
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]
    n_test = min(wl.n, 262144)
    X = workloads.make_X(wl.with_rows(max(n_test, wl.B)), dev)
    idx = workloads.landmark_indices(wl.with_rows(max(n_test, wl.B)))
    L = X[idx.to(dev)].contiguous()
    Xt = X[:n_test]
    t0 = time.perf_counter()
    if args.random_w:
        W_host = torch.randn((wl.B, wl.B), generator=torch.Generator().manual_seed(1)) / wl.B ** 0.5
        rank = wl.B
    else:
        W_host, rank = whiten(args, lpd, L, wl.gamma)
    t_whiten = time.perf_counter() - t0
    c = args.classifiers
    Ws = (torch.randn((c, rank), generator=torch.Generator().manual_seed(2)) / rank ** 0.5)
    W = W_host.to(dev)
    V = lpd.lpd_fold_weights(W, Ws.to(dev), r=rank)
    F = torch.empty((n_test, c), dtype=torch.float32, device=dev)
    ws = lpd.alloc_workspace(n_test, wl.d, wl.B, dev)
    evs = []

    def step(collect):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        lpd.lpd_predict(Xt, L, wl.gamma, V, F, ws)
        e1.record()
        if collect:
            evs.append((e0, e1))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
    flop = 2.0 * n_test * wl.B * (wl.d + (c if c > 32 else 0))
    tflops = flop / (ms * 1e-3) / 1e12
    out = {
        "metric": "prediction_rows_per_s", "value": n_test * len(evs) / elapsed, "unit": "rows/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / len(evs),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" + (" (random W: tuning run)" if args.random_w else ""),
        "config": {"workload": wl.name + " (first rows as new points)", "n_test": n_test, "d": wl.d, "B": wl.B,
                   "rank": rank, "classifiers": c, "gamma": wl.gamma},
        "whiten_s": None if args.random_w else t_whiten,
        "roofline": {"kernel": ("lpd_predict: gemm_nt_kernel<EPI_GAUSS_DOT> (kernel block contracted with the folded weights "
                                "in its own launch) + the pass that adds the tile columns' shares" if c <= 64 else
                                "lpd_predict: gemm_nt_kernel<EPI_GAUSS> panels + MFMA product with the folded weights"),
                     "bound": "mfma",
                     "achieved": tflops, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP32_MFMA_PEAK_TFLOPS, "flop_per_launch": flop, "avg_launch_ms": ms,
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import lpd_oracle as orc
        Xs = Xt[: 1 << 14].cpu().numpy()
        Lh, Wh, Wsh = L.cpu().numpy(), W_host[:rank].numpy(), Ws.numpy()
        probe = 32
        t0 = time.perf_counter()
        orc.predict(Xs[:probe], Lh, wl.gamma, Wh, Wsh, r=rank)
        per_row = (time.perf_counter() - t0) / probe
        m = int(max(probe, min(Xs.shape[0], args.cpu_seconds / max(per_row, 1e-9))))
        t0 = time.perf_counter()
        orc.predict(Xs[:m], Lh, wl.gamma, Wh, Wsh, r=rank)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": m / t_cpu, "unit": "rows/s", "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {m} of the {n_test} new points, all {wl.B} landmarks, "
                                         f"{c} classifiers, double precision, {t_cpu:.1f} s",
                               "gpu_over_cpu": out["value"] / (m / t_cpu)}
    print(json.dumps(out))


def bench_stream(args):
    """Step 1d streamed to pinned host memory: device compute overlapped with the copy of G over PCIe."""
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    t0 = time.perf_counter()
    if args.random_w:
        W_host = torch.randn((wl.B, wl.B), generator=torch.Generator().manual_seed(1)) / wl.B ** 0.5
        rank = wl.B
    else:
        W_host, rank = whiten(args, lpd, L, wl.gamma)
    t_whiten = time.perf_counter() - t0
    W = W_host.to(dev)
    chunk_rows, nbytes = lpd.lpd_nystrom_factor_to_host_workspace(wl.n, wl.d, wl.B, args.chunk_rows)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    t0 = time.perf_counter()
    G_host = torch.empty((wl.n, wl.B), dtype=torch.float32, pin_memory=True)
    t_pin = time.perf_counter() - t0
    for _ in range(args.warmup):
        lpd.lpd_nystrom_factor_to_host(X, L, wl.gamma, W, G_host, chunk_rows, ws, r=rank)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        lpd.lpd_nystrom_factor_to_host(X, L, wl.gamma, W, G_host, chunk_rows, ws, r=rank)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = elapsed * 1e3 / args.steps
    flop = 2.0 * wl.n * wl.B * (wl.d + rank)
    tflops = flop / (ms * 1e-3) / 1e12
    out = {
        "metric": "stage1_factor_rows_per_s_to_host", "value": wl.n * args.steps / elapsed, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" + (" (random W: tuning run)" if args.random_w else ""),
        "config": {"workload": wl.name, "n": wl.n, "d": wl.d, "B": wl.B, "rank": rank, "gamma": wl.gamma,
                   "chunk_rows": chunk_rows, "workspace_bytes": nbytes, "G_host": "pinned, n x B float32"},
        "whiten_s": None if args.random_w else t_whiten, "pin_alloc_s": t_pin,
        "pcie_GBps": wl.n * wl.B * 4 / (ms * 1e-3) / 1e9,
        "roofline": {"kernel": "lpd_nystrom_factor_to_host: both GEMMs per chunk, copy of G overlapped",
                     "bound": "mfma", "achieved": tflops, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP32_MFMA_PEAK_TFLOPS, "flop_per_launch": flop, "avg_launch_ms": ms,
                     "traffic": None},
    }
    print(json.dumps(out))


def bench_whiten(args):
    """Steps 1a-1c on the device for the workload's landmarks: seconds per preparation, phase by phase."""
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]
    n_rows = max(4 * wl.B, 65536)                 # landmarks are drawn from the first rows of the recipe
    wl_s = wl.with_rows(min(wl.n, n_rows))
    X = workloads.make_X(wl_s, dev)
    L = X[workloads.landmark_indices(wl_s).to(dev)].contiguous()
    del X
    B = wl.B
    ws = torch.empty(lpd.lpd_whiten_workspace(B), dtype=torch.uint8, device=dev)
    for _ in range(args.warmup):
        lpd.lpd_whiten(L, wl.gamma, workspace=ws)
    phases, totals = {}, []
    for _ in range(args.steps):
        ph = {}
        t0 = time.perf_counter()
        W, eig, rank = lpd.lpd_whiten(L, wl.gamma, workspace=ws, phases=ph)
        totals.append(time.perf_counter() - t0)
        for k, v in ph.items():
            phases[k] = phases.get(k, 0.0) + v / args.steps
    sec = sum(totals) / len(totals)
    # matrix-vector pass of column j: the upper triangle of the m x m trailing matrix read once, m = B - j - 1
    bytes_trail = 4.0 * sum(float(m) * (m + 1) for m in range(2, B))
    gbps = bytes_trail / max(phases["tridiagonalisation"], 1e-9) / 1e9
    out = {
        "metric": "stage1_preparation_seconds", "value": sec, "unit": "s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": wl.name + " (landmarks only)", "B": B, "d": wl.d, "gamma": wl.gamma, "rank": rank,
                   "workspace_bytes": ws.numel()},
        "phases_s": phases,
        "roofline": {"kernel": "symv_upper_kernel (upper triangle of the trailing matrix times reflector, one read-only "
                               "pass per column); time = the whole tridiagonalisation phase, panel updates and the small "
                               "per-column kernels included",
                     "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "bytes_per_call": bytes_trail, "traffic": None,
                     "note": "a pass over the whole symmetric matrix, which the first version of this routine made, "
                             "would be priced at twice these bytes"},
    }
    if not args.no_cpu_baseline and B <= 4096:
        t0 = time.perf_counter()
        lpd.lpd_whiten_host(L.cpu(), wl.gamma)
        out["host_routine_s"] = time.perf_counter() - t0
    print(json.dumps(out))


def bench_sparse(args):
    """Step 1d with X in compressed-row form (default: the 80 %-zeros 'digit' recipe)."""
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]
    if args.density is not None:
        wl = wl.with_density(args.density)
    lpd.lpd_set_option(lpd.LPD_OPT_CSR_ROUTE, lpd.CSR_ROUTES[args.csr_route])
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    t0 = time.perf_counter()
    if args.random_w:
        W_host = torch.randn((wl.B, wl.B), generator=torch.Generator().manual_seed(1)) / wl.B ** 0.5
        rank = wl.B
    else:
        W_host, rank = whiten(args, lpd, L, wl.gamma)
    t_whiten = time.perf_counter() - t0
    W = W_host.to(dev)
    rp, ci, va = workloads.to_csr(X)
    nnz = int(ci.numel())
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    # the dense factor on the same rows, for comparison
    ws_d = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev)
    lpd.lpd_nystrom_factor(X, L, wl.gamma, W, G, ws_d, r=rank)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    lpd.lpd_nystrom_factor(X, L, wl.gamma, W, G, ws_d, r=rank)
    e1.record()
    torch.cuda.synchronize()
    ms_dense = e0.elapsed_time(e1)
    del X, ws_d
    chunk_rows, nbytes = lpd.lpd_nystrom_factor_csr_workspace(wl.n, wl.d, wl.B, args.chunk_rows, nnz)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    route = args.csr_route if args.csr_route != "auto" else ("gather" if nnz < 0.08 * wl.n * wl.d else "dense")
    evs = []
    for i in range(args.warmup + args.steps):
        if i == args.warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        lpd.lpd_nystrom_factor_csr(rp, ci, va, wl.d, L, wl.gamma, W, G, chunk_rows, ws, r=rank, validate=i == 0)
        b.record()
        if i >= args.warmup:
            evs.append((a, b))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
    flop = 2.0 * wl.n * wl.B * (wl.d + rank)
    tflops = flop / (ms * 1e-3) / 1e12
    out = {
        "metric": "nystrom_factor_rows_per_s_from_csr", "value": wl.n * args.steps / elapsed, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" + (" (random W: tuning run)" if args.random_w else ""),
        "config": {"workload": wl.name + " (X in compressed-row form)", "n": wl.n, "d": wl.d, "B": wl.B, "rank": rank,
                   "gamma": wl.gamma, "nnz": nnz, "density": nnz / (wl.n * wl.d), "route": route,
                   "chunk_rows": chunk_rows,
                   "x_bytes_csr": 12 * nnz + 8 * (wl.n + 1), "x_bytes_dense": 4 * wl.n * wl.d},
        "ms_dense_factor_same_rows": ms_dense,
        "whiten_s": None if args.random_w else t_whiten,
        "roofline": {"kernel": "lpd_nystrom_factor_csr (" + route + " route), then the whitening product; "
                               "flops counted as for the dense products, 2 n B (d + r)",
                     "bound": "mfma", "achieved": tflops, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP32_MFMA_PEAK_TFLOPS, "flop_per_launch": flop, "avg_launch_ms": ms,
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import lpd_oracle as orc
        m = 256
        t0 = time.perf_counter()
        r0, r1 = int(rp[0]), int(rp[m])
        sub = (rp[: m + 1] - rp[0]).cpu().numpy(), ci[r0:r1].cpu().numpy(), va[r0:r1].cpu().numpy()
        Zs = orc.kernel_block_csr(*sub, wl.d, L.cpu().numpy(), wl.gamma)
        orc.apply_whitening(Zs, W_host.numpy(), rank)
        per_row = (time.perf_counter() - t0) / m
        m2 = int(max(m, min(16384, args.cpu_seconds / max(per_row, 1e-9))))
        r1 = int(rp[m2])
        sub = (rp[: m2 + 1] - rp[0]).cpu().numpy(), ci[:r1].cpu().numpy(), va[:r1].cpu().numpy()
        t0 = time.perf_counter()
        Zs = orc.kernel_block_csr(*sub, wl.d, L.cpu().numpy(), wl.gamma)
        orc.apply_whitening(Zs, W_host.numpy(), rank)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": m2 / t_cpu, "unit": "rows/s", "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"first {m2} of {wl.n} rows, all {wl.B} landmarks, double precision, "
                                         f"{t_cpu:.1f} s", "gpu_over_cpu": out["value"] / (m2 / t_cpu)}
    print(json.dumps(out))


def bench_calibrate(args):
    """A copy of known size for scaling the traffic counters: 1 GiB read, 1 GiB written, args.steps times."""
    import torch
    dev = torch.device("cuda:0")
    n = 1 << 28
    src = torch.ones(n, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dst.copy_(src)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    print(json.dumps({"metric": "copy_GBps", "value": 2.0 * 4 * n / sec / 1e9, "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n,
                      "kib_per_copy_each_way": 4 * n // 1024}))


def bench_multi(args):
    """Margins of --vectors weight vectors at once (folds, C values, class pairs sharing one G): one pass of
    lpd_margins_multi over a synthetic G of the workload's shape (rows capped at 32 GiB of G)."""
    import torch
    from paper_2207_01016_amd import lpd, workloads
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]
    r = wl.B
    n = min(wl.n, (32 << 30) // (4 * r))
    g = torch.Generator(device=dev).manual_seed(5)
    G = torch.randn((n, r), generator=g, device=dev)
    k = args.vectors
    Ws = torch.randn((k, r), generator=g, device=dev) / r ** 0.5
    M = torch.empty((n, k), dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        lpd.lpd_margins_multi(G, Ws, M)
    evs = []
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        lpd.lpd_margins_multi(G, Ws, M)
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
    gbps = 4.0 * n * r / ms / 1e6
    tflops = 2.0 * n * r * k / ms / 1e9
    print(json.dumps({"metric": "multi_vector_sweep_rows_per_s", "value": n / ms * 1e3, "unit": "rows/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                      "dtype": "f32", "data": "synthetic",
                      "config": {"workload": args.workload, "rows": n, "r": r, "vectors": k},
                      "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                   "frac": gbps / HBM_PEAK_GBPS, "traffic": None,
                                   "kernel": "one pass over G (4 n r bytes)"},
                      "mfma_tflops": tflops, "mfma_frac_of_fp32_peak": tflops / FP32_MFMA_PEAK_TFLOPS}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2207_01016_amd import lpd, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    lpd.lib()
    if args.path == "solver":
        bench_solver(args)
        return
    if args.path == "predict":
        bench_predict(args)
        return
    if args.path == "stream":
        bench_stream(args)
        return
    if args.path == "whiten":
        bench_whiten(args)
        return
    if args.path == "sparse":
        bench_sparse(args)
        return
    if args.path == "multi":
        bench_multi(args)
        return
    if args.path == "calibrate":
        bench_calibrate(args)
        return
    dev = torch.device("cuda:0")
    wl = workloads.WORKLOADS[args.workload]

    # ---- inputs, resident in HBM
    X = workloads.make_X(wl, dev)
    idx = workloads.landmark_indices(wl)
    L = X[idx.to(dev)].contiguous()
    L_host = L.cpu()
    t0 = time.perf_counter()
    if args.random_w:
        g = torch.Generator().manual_seed(1)
        W_host = torch.randn((wl.B, wl.B), generator=g) / wl.B ** 0.5
        rank = wl.B
    else:
        W_host, rank = whiten(args, lpd, L, wl.gamma)
    t_whiten = time.perf_counter() - t0
    W = W_host.to(dev)
    w = workloads.make_w(wl).to(dev)
    G = torch.empty((wl.n, wl.B), dtype=torch.float32, device=dev)
    m = torch.empty(wl.n, dtype=torch.float32, device=dev)
    rec, mn = lpd.lpd_nystrom_factor_workspace(wl.n, wl.d, wl.B)
    ws_bytes = int(rec * args.workspace_mult)
    if args.panel_rows > 0:
        # bytes per panel row from the two sizes the query reports (minimum: 256 rows; recommended: rec_rows rows)
        ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev, rec)
        rec_rows = lpd.lpd_nystrom_factor_profiled(X, L, wl.gamma, W, G, ws, r=rank).panel_rows
        del ws
        row_bytes = (rec - mn) / max(rec_rows - 256, 1)
        ws_bytes = int(mn + (args.panel_rows - 256 + 0.5) * row_bytes)
    ws = lpd.alloc_workspace(wl.n, wl.d, wl.B, dev, ws_bytes)
    lpd.lpd_set_option(lpd.LPD_OPT_GEMM_TILE, lpd.GEMM_TILES[args.tile])

    def step(collect):
        prof = lpd.lpd_nystrom_factor_profiled(X, L, wl.gamma, W, G, ws, r=rank)   # blocks; events per launch
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        lpd.lpd_margins(G, w, m, r=rank)
        e1.record()
        if collect is not None:
            collect.append((prof, e0, e1))

    t0 = time.perf_counter()
    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    warm_ms = (time.perf_counter() - t0) * 1e3 / args.warmup if args.warmup > 0 else float("inf")
    # A step of a few milliseconds or less is dominated by what the profiled call adds on the host (two events
    # per launch, a blocking read-out per step).  Such workloads are timed through the plain, enqueue-only calls
    # (events around the factor and around the sweep of every step, one synchronisation at the end), and the
    # split over the kernels comes from the same number of profiled steps run right after, outside `value`.
    plain_timing = warm_ms < 20.0
    records = []
    if plain_timing:
        marks = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            ev[0].record()
            lpd.lpd_nystrom_factor(X, L, wl.gamma, W, G, ws, r=rank)
            ev[1].record()
            lpd.lpd_margins(G, w, m, r=rank)
            ev[2].record()
            marks.append(ev)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        for _ in range(args.steps):
            step(records)
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(records)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

    steps = max(args.steps, 1)
    ms_step = elapsed * 1e3 / steps
    ms_whiten = sum(p.ms_whiten for p, _, _ in records)
    ms_kb = sum(p.ms_kernel_block for p, _, _ in records)
    ms_norms = sum(p.ms_norms for p, _, _ in records)
    launches = sum(p.launches_whiten for p, _, _ in records)
    ms_sweep = sum(a.elapsed_time(b) for _, a, b in records)
    ms_factor = ms_whiten + ms_kb + ms_norms
    if plain_timing:
        ms_factor = sum(ev[0].elapsed_time(ev[1]) for ev in marks)    # whole factor call, gaps between launches included
        ms_sweep = sum(ev[1].elapsed_time(ev[2]) for ev in marks)

    flop_factor = 2.0 * wl.n * wl.B * (wl.d + rank)
    # few landmarks: one launch does the kernel block and the whitening product (booked under "whiten")
    one_launch = bool(records) and records[0][0].launches_kernel_block == 0
    flop_dominant = flop_factor if one_launch else 2.0 * wl.n * wl.B * rank
    flop_whiten_launch = flop_dominant * steps / max(launches, 1)
    whiten_tflops = flop_dominant * steps / (ms_whiten * 1e-3) / 1e12
    factor_tflops = flop_factor * steps / (ms_factor * 1e-3) / 1e12
    sweep_bytes = 4.0 * wl.n * rank
    sweep_gbps = sweep_bytes * steps / (ms_sweep * 1e-3) / 1e9

    panel_rows = records[0][0].panel_rows if records else None
    traffic_dominant, traffic_sweep = measured_traffic(wl.name, panel_rows)
    out = {
        "metric": "nystrom_factor_plus_margin_sweep_rows_per_s",
        "value": wl.n * steps / elapsed,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic" + (" (random W: tuning run, not a valid measurement)" if args.random_w else ""),
        "config": {"workload": wl.name, "n": wl.n, "d": wl.d, "B": wl.B, "rank": rank, "gamma": wl.gamma,
                   "panel_rows": panel_rows, "gemm_tile": args.tile,
                   "choice": "largest of BASELINE.json's five configurations (all fit one GPU, its metric names none)"
                             if wl.name == "highrank" else "selected with --workload"},
        "factor": {"ms_per_step": ms_factor / steps, "rows_per_s": wl.n * steps / (ms_factor * 1e-3),
                   "tflops": factor_tflops, "frac_of_fp32_mfma_peak": factor_tflops / FP32_MFMA_PEAK_TFLOPS,
                   "ms_kernel_block": ms_kb / steps, "ms_whiten": ms_whiten / steps, "ms_norms": ms_norms / steps},
        "sweep": {"ms_per_step": ms_sweep / steps, "gbps": sweep_gbps, "frac_of_hbm_peak": sweep_gbps / HBM_PEAK_GBPS},
        "whiten_s": None if args.random_w else t_whiten, "whiten_routine": None if args.random_w else args.whiten,
        "timing": ("plain enqueue-only calls in the timed steps (events around the factor and the sweep); the "
                   "per-kernel figures below come from as many profiled steps run right after")
                  if plain_timing else "profiled calls in the timed steps (HIP events around every launch)",
        "roofline": {"kernel": "nystrom_small_kernel (kernel block and whitening product in one launch, Z in LDS)"
                               if one_launch else "gemm_nt_kernel<EPI_STORE> (whitening product Z W^T)", "bound": "mfma",
                     "achieved": whiten_tflops, "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": whiten_tflops / FP32_MFMA_PEAK_TFLOPS,
                     "flop_per_launch": flop_whiten_launch, "avg_launch_ms": ms_whiten / max(launches, 1),
                     "launches": launches, "traffic": traffic_dominant},
        "roofline_sweep": {"kernel": "margins_kernel", "bound": "hbm", "achieved": sweep_gbps, "peak": HBM_PEAK_GBPS,
                           "unit": "GB/s", "frac": sweep_gbps / HBM_PEAK_GBPS, "bytes_per_launch": sweep_bytes,
                           "avg_launch_ms": ms_sweep / steps, "traffic": traffic_sweep},
    }

    if not args.no_cpu_baseline:
        from oracle import lpd_oracle as orc
        Xs = X[: min(wl.n, 1 << 16)].cpu().numpy()   # the baseline picks how many of these it needs
        out["cpu_baseline"] = cpu_baseline(orc, wl, Xs, L_host.numpy(), W_host[:rank].numpy(), w[:rank].cpu().numpy(),
                                           args.cpu_seconds)
        out["cpu_baseline"]["gpu_over_cpu"] = out["value"] / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
