#!/usr/bin/env python3
"""Benchmark of the batch-SOM epoch on one MI355X.

A step = one whole training epoch (`som_train_epoch_dense`: BMU search + batch update) over
the configuration-2 workload (dense fp32, n = 100,000, dim = 1,000, 50x50 toroid square map),
with the data already resident in HBM.  Step s runs epoch s mod 10 of the linear radius
schedule 25 -> 1; whenever the schedule restarts, the code book is reset to its seeded initial
value (a device copy inside the timed region).  Prints ONE JSON line.

`--workload 5|3|1` times another dense configuration, `--workload 4` the sparse one, `--workload
6|7` two further sparse shapes of the paper's own experiments; the default line is
configuration 2, the one the metric is quoted on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "epoch throughput (instance*node*dim/s)"
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_FP16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel (fetched + written), from the rocprofv3 --pmc passes
# (FETCH_SIZE, WRITE_SIZE, scaled by the copy calibration) summarised in profiles/epoch_config*.md;
# measured once per kernel version, not during this run (the dense figures vary by some ten percent from
# run to run: they depend on how long the workgroups that share an instance tile stay in step).
MEASURED_TRAFFIC_BYTES = {(2, "two_level"): 1.388e9 + 0.034e9, (3, "two_level"): 2.906e9 + 0.094e9,
                          (5, "two_level"): 4.446e9 + 0.424e9,
                          (6, "two_level"): 2.977e9 + 0.035e9,      # sparse rows searched through dense planes
                          # one-level split-fp16 filter and fp32 filter (earlier counter runs; those kernels are unchanged)
                          (2, "split_f16"): 3.841e9 + 0.036e9, (2, "fp32"): 8.49e9 + 0.025e9,
                          (3, "split_f16"): 14.283e9 + 0.025e9, (5, "split_f16"): 13.917e9 + 0.072e9,
                          # sparse: all kernels of the filter stage (code-book pass, hot-column block, sweep)
                          (4, "sparse"): 16.393e9 + 1.453e9, (6, "sparse"): 0.415e9 + 0.058e9,
                          (7, "sparse"): 87.465e9 + 6.475e9}
PEAK_FP32_VALU_TFLOPS = 157.3


def cpu_baseline(w, X, W0, seconds_budget: float = 20.0):
    """The oracle, as it stands, on a bounded sample of the same workload: one whole epoch
    (BMU search + update of the full map) over the first n_s instances."""
    from oracle import som_oracle as oracle
    cores = oracle.num_threads()
    mt, gt = oracle.MAP_TYPES[w.map_type], oracle.GRID_TYPES[w.grid_type]
    # ~1.5e9 instance*node*dim per second and core is what the plain fp64 loop reaches
    per_s = 1.0e9 * cores
    n_s = int(max(64, min(w.n, seconds_budget * per_s / (w.k * (w.dim if w.kind == "dense" else w.dim)))))
    t0 = time.perf_counter()
    if w.kind == "dense":
        oracle.epoch_dense(X[:n_s], W0, w.rows, w.cols, mt, gt, w.radius0)
    else:
        indptr, indices, values = X
        sub = (indptr[: n_s + 1].copy(), indices[: indptr[n_s]], values[: indptr[n_s]])
        oracle.epoch_csr(sub, w.dim, W0, w.rows, w.cols, mt, gt, w.radius0)
    dt = time.perf_counter() - t0
    return {"value": n_s * w.k * w.dim / dt, "unit": "instance*node*dim/s", "cores": cores, "kind": "oracle",
            "sample": f"one whole oracle epoch (BMU + update, radius {w.radius0:g}) over the first {n_s} of "
                      f"{w.n} instances, full {w.rows}x{w.cols} map, {dt:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5, 6, 7])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--filter", choices=["auto", "two_level", "split_f16", "fp32"], default="auto",
                    help="arithmetic of the dense BMU filter pass (same BMUs either way)")
    ap.add_argument("--neighborhood", choices=["gaussian", "gaussian-compact", "bubble"], default="gaussian",
                    help="neighbourhood of the update (the stated configurations use the plain Gaussian)")
    ap.add_argument("--smoothing", choices=["auto", "vector", "matrix", "matrix_split"], default="auto",
                    help="units that run the Gaussian smoothing passes (same results)")
    ap.add_argument("--mode", choices=["epoch", "map"], default="epoch",
                    help="epoch (default): a step is one training epoch of the schedule.  map: the schedule is "
                         "trained once, untimed, and a step is one BMU search (som_bmus_*) of the whole data set "
                         "against that trained map - the post-training mapping, a slow corner of the exact stage")
    ap.add_argument("--no-hot-block", action="store_true",
                    help="sparse workloads: keep all columns in the gather sweep (no dense block of frequent columns)")
    ap.add_argument("--no-dense-planes", action="store_true",
                    help="sparse workloads of modest dimension: keep the gather sweep (no dense filter pass on planes)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run ten plain 1 GiB device copies and exit: under rocprofv3 --pmc this gives the "
                         "reading of FETCH_SIZE / WRITE_SIZE for a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from gen import make_workload
    from paper_1305_1422_amd import Som, capi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": src.numel() * 4,
                                               "bytes_written_per_copy": src.numel() * 4, "copies": 10}}))
        return 0

    w = make_workload(args.workload)
    X = w.data()
    W0 = w.codebook()
    dev = torch.device("cuda:0")
    if w.kind == "dense":
        Xd = torch.from_numpy(X).to(dev)
    else:
        Xd = tuple(torch.from_numpy(a).to(dev) for a in X)
    W0d = torch.from_numpy(W0).to(dev)
    som = Som(w.rows, w.cols, w.dim, w.map_type, w.grid_type, codebook=W0d, filter=args.filter)
    if args.neighborhood != "gaussian":
        som.set_neighborhood("bubble" if args.neighborhood == "bubble" else "gaussian", args.neighborhood != "bubble")
    som.set_smoothing(args.smoothing)
    if args.no_hot_block:
        som.set_sparse_hot_block(False)
    if args.no_dense_planes:
        som.set_sparse_dense_filter(False)
    bmus = torch.empty(w.n, dtype=torch.int32, device=dev)
    # register the resident training set: its norms are then computed once, not every epoch
    if w.kind == "dense":
        capi.som_set_data_dense(som.ctx, Xd)
    else:
        capi.som_set_data_csr(som.ctx, *Xd)
    radii = [w.radius0 + (w.radiusN - w.radius0) * e / max(1, w.epochs - 1) for e in range(w.epochs)]

    if args.mode == "map":
        for e in range(w.epochs):
            som.train_epoch(Xd, radii[e], 1.0, bmus)

    def step(s: int):
        if args.mode == "map":
            som.bmus(Xd, bmus)
            return
        e = s % w.epochs
        if e == 0:
            som.codebook.copy_(W0d)
        som.train_epoch(Xd, radii[e], 1.0, bmus)

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    capi.som_profile_enable(som.ctx, True)
    capi.som_profile_read(som.ctx)          # clear
    # one event per step on the stream the library launches on (torch's current stream): the
    # per-epoch figures below come from these, the headline value from the host clock around the
    # whole timed region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        marks[s].record()
        step(args.warmup + s)
    marks[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_epoch = [[] for _ in range(w.epochs)]
    for s in range(args.steps):
        per_epoch[(args.warmup + s) % w.epochs].append(marks[s].elapsed_time(marks[s + 1]))
    epoch_ms_median = [float(np.median(v)) if v else None for v in per_epoch]
    prof = capi.som_profile_read(som.ctx)
    capi.som_profile_enable(som.ctx, False)
    refined, collected, rescanned = som.stats()

    # two-level dense search: share of the (instance tile, node block) pairs its second pass works on, from one
    # more, untimed, run through the schedule (the call that reads it synchronises)
    fine_share = None
    planes = w.kind != "dense" and capi.som_sparse_dense_filter_active(som.ctx)    # sparse rows, dense filter pass
    if (w.kind == "dense" or planes) and args.mode == "epoch":
        shares = []
        for e in range(w.epochs):
            step(e)
            listed, pairs = som.two_level_stats()
            if pairs:
                shares.append(listed / pairs)
        if shares:
            fine_share = {"mean": float(np.mean(shares)), "per_epoch": [round(v, 4) for v in shares]}

    ms_per_step = 1e3 * dt / args.steps
    work = float(w.n) * w.k * w.dim
    value = work / (dt / args.steps)

    stage_ms = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}
    if w.kind == "dense" or planes:
        dom_ms = stage_ms["bmu_csr_filter" if planes else "bmu_dense_filter"]
        flops = 2.0 * work                               # one multiply-add per (instance, node, feature)
        fp32_equiv = flops / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
        # achieved = the method's own work, one multiply-add per (instance, node, feature) = 2 n k dim flop,
        # over the kernel's launch time, against the dense peak of the matrix format the contraction runs in
        if args.filter == "fp32":
            roofline = {"bound": "mfma", "kernel": "k_bmu_dense_dl<false> (fp32 MFMA BMU filter pass)",
                        "achieved": fp32_equiv, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": fp32_equiv / PEAK_FP32_MFMA_TFLOPS,
                        "traffic": MEASURED_TRAFFIC_BYTES.get((w.config, args.filter)), "avg_launch_ms": dom_ms}
        elif fine_share is not None:
            # two-level search: one fp16 product per (instance, node, feature) in the coarse pass and three
            # more on the share of the pairs the second pass works on: mfma_issue_frac counts those (how busy
            # the matrix pipe is), frac counts the method's one multiply-add per triple.  avg_launch_ms is the
            # whole filter stage (coarse pass, block selection, ordering, lists, second pass)
            products = 1.0 + 3.0 * fine_share["mean"]
            roofline = {"bound": "mfma", "kernel": "two-level BMU filter stage: k_bmu_coarse (block minima, 1 fp16 product) + "
                                                   "k_select_blocks + radix sort + k_tile_lists + k_bmu_dense_h<fine, 3 fp16 "
                                                   "products on the listed pairs>",
                        "achieved": fp32_equiv, "peak": PEAK_FP16_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": fp32_equiv / PEAK_FP16_MFMA_TFLOPS,
                        "traffic": MEASURED_TRAFFIC_BYTES.get((w.config, "two_level")), "avg_launch_ms": dom_ms,
                        "second_pass_share_of_pairs": fine_share,
                        "mfma_issue_frac": products * fp32_equiv / PEAK_FP16_MFMA_TFLOPS,
                        "vs_fp32_mfma_peak": fp32_equiv / PEAK_FP32_MFMA_TFLOPS}
        else:
            # the kernel issues three fp16 matrix products per (instance, node, feature), hi*hi + hi*lo + lo*hi:
            # mfma_issue_frac counts those (how busy the matrix pipe is), frac does not
            roofline = {"bound": "mfma", "kernel": "k_bmu_dense_h<2, 0> (BMU filter pass, 3 fp16 MFMAs on split fp32 operands)",
                        "achieved": fp32_equiv, "peak": PEAK_FP16_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": fp32_equiv / PEAK_FP16_MFMA_TFLOPS,
                        "traffic": MEASURED_TRAFFIC_BYTES.get((w.config, args.filter)), "avg_launch_ms": dom_ms,
                        "mfma_issue_frac": 3.0 * fp32_equiv / PEAK_FP16_MFMA_TFLOPS,
                        "vs_fp32_mfma_peak": fp32_equiv / PEAK_FP32_MFMA_TFLOPS}
        if planes:
            roofline["note"] = ("sparse rows of modest dimension: the filter pass runs on dense fp16 planes of the centred rows "
                                "(som_set_sparse_dense_filter), priced as n*k*dim multiply-adds like the dense workloads; "
                                "the exact stage and the update work on the sparse rows")
    else:
        indptr = X[0]
        nnz = int(indptr[-1])
        dom_ms = stage_ms["bmu_csr_filter"]
        # compulsory bytes: CSR once (8 B per nonzero + 8 B per row), code book once, BMUs out
        alg_bytes = nnz * 8.0 + (w.n + 1) * 8.0 + w.k * w.dim * 4.0 + w.n * 4.0
        achieved = alg_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
        traffic = MEASURED_TRAFFIC_BYTES.get((w.config, "sparse"))
        valu_bound_ms = 2.0 * nnz * w.k / (PEAK_FP32_VALU_TFLOPS * 1e12) * 1e3
        roofline = {"bound": "hbm", "kernel": "sparse BMU filter pass: k_center_transpose_q16 + hot-column block "
                                              "(k_bmu_dense_h<partial>) + k_bmu_csr_sliced",
                    "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                    "traffic": traffic, "avg_launch_ms": dom_ms,
                    # the three views of this kernel: (i) against the plain fp32 vector ALUs, on which 2 nnz k
                    # flop cannot take less than valu_bound_ms; (ii) `frac` above: compulsory bytes (CSR once,
                    # code book once, BMUs) against the HBM peak; (iii) the traffic the gathers really send past
                    # L2 (counter readings of the stage's kernels, with the hot-column block on) against the HBM peak
                    "valu_bound_ms": valu_bound_ms, "frac_of_valu_bound": valu_bound_ms / dom_ms if dom_ms > 0 else None,
                    "compulsory_bytes": alg_bytes,
                    "traffic_rate_gbs": traffic / (dom_ms * 1e-3) / 1e9 if traffic and dom_ms > 0 else None,
                    "traffic_frac_of_hbm_peak": (traffic / (dom_ms * 1e-3) / 1e9 / PEAK_HBM_GBS
                                                 if traffic and dom_ms > 0 else None)}

    out = {
        "metric": METRIC, "value": value, "unit": "instance*node*dim/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f32" if (w.kind != "dense" and not planes) or args.filter == "fp32" else
                  "f32 operands split into 2 x f16, f32 accumulation (filter); f64 (decision)"),
        "data": "synthetic",
        "config": {"workload": f"config {w.config}: {w.name}", "kind": w.kind, "n": w.n, "dim": w.dim,
                   "map": f"{w.rows}x{w.cols} {w.map_type} {w.grid_type}",
                   "schedule": f"radius {w.radius0:g}->{w.radiusN:g} linear over {w.epochs} epochs, step s = epoch s mod {w.epochs}",
                   "mode": args.mode,
                   "step": ("som_bmus on the registered data set against the map the schedule has trained: BMU search alone"
                            if args.mode == "map" else
                            "som_train_epoch on the registered data set: BMU search + batch update, everything that "
                            "depends on the code book included; outside the step, once per registered data set: "
                            + ("squared norms of the instances, their fp16 hi/lo planes, sampled column means"
                               if w.kind == "dense" else
                               "column means, squared norms and fp16 hi/lo planes of the centred rows" if planes else
                               "squared norms of the instances, hot-column split")),
                   "neighborhood": args.neighborhood, "smoothing": args.smoothing,
                   "sparse_hot_block": bool(w.kind != "dense" and capi.som_sparse_hot_block_active(som.ctx)),
                   "sparse_dense_planes": bool(w.kind != "dense" and capi.som_sparse_dense_filter_active(som.ctx))},
        "gflops_epoch": 2.0 * work / (dt / args.steps) / 1e9,
        "frac_fp32_mfma_peak_whole_epoch": 2.0 * work / (dt / args.steps) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "stage_ms": stage_ms,
        "epoch_ms_median": epoch_ms_median,      # by position in the radius schedule (epoch 0 = widest radius)
        "last_step_exact_rows": {"refined": refined, "collected": collected, "rescanned": rescanned},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, X, W0)
    som.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
