#!/usr/bin/env python3
"""Throughput benchmark of the PR-SGD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5] [--interval I]

A step is one iteration of Algorithm 1 over all N workers: seeded minibatch draw, forward,
backward, local update (eq. 3), plus the restart average (eq. 2) after every I-th
iteration.  The default workload is the largest configuration (c5: N = 8 replicas of a
4096-4096-4096-4096-1000 ReLU MLP, bf16 matrix operands, B = 128, I = 16), the one whose replica
set is far larger than the caches.  Inputs are synthetic and resident in HBM before the timed
region.  Prints ONE JSON line: samples/s over the N replicas, a roofline record for the kernel
that dominates the step, the restart-average and stand-alone update bandwidths at HBM scale, and
the CPU oracle timed on a bounded sample of the same workload as a reported baseline.
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

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

# rocprofv3 kernel symbol behind each timing label of the library
KERNEL_SYMBOL = {
    "gather": "gather_kernel", "gemm_fwd": "grouped_gemm_kernel<.., OP_CONTIG, OP_TRANS>",
    "gemm_dx": "grouped_gemm_kernel<.., OP_CONTIG, OP_CONTIG>",
    "gemm_dw": "grouped_gemm_kernel<.., OP_TRANS, OP_TRANS>",
    "gemm_bwd": "grouped_bwd_full_kernel (grouped_bwd_kernel for layers with partial tiles)",
    "softmax_xent": "softmax_xent_kernel (loss head + row gather of the next iteration)",
    "sgd_update": "update_kernel",
    "average": "average_kernel (restart_small_kernel<.., true> when N >= 8 and a replica has fewer "
               "than 262144 floats)",
    "restart_mean": "mean_kernel (restart_small_kernel<.., false> when N >= 8 and a replica has "
                    "fewer than 262144 floats)",
    "lsq_steps": "lsq_steps_staged_kernel (lsq_steps_kernel for shapes it does not take)",
    "mlp2_epoch": "mlp2_epoch_kernel",
    "gemm_bwd_first": "bwd_first_fwd_kernel (layer 1: backward step + next forward product)",
    "refresh_shadow": "refresh_shadow_kernel (bf16 image of W_1 when the first-layer chain breaks)",
    "step_mean": "grouped_gemm_kernel<.., OP_TRANS, OP_TRANS, true> (the minibatches of all workers "
                 "stacked into one contraction)",
}


def algorithmic_work(w, shared_weights=False, first_fused=False):
    """Algorithmic HBM bytes and flops of ONE iteration, per kernel label (all launches of
    that label in the iteration summed), plus those of one restart average.  shared_weights:
    every iteration starts from the node average (I = 1, one-pass form), so the forward and
    backward-data products read one weight matrix per layer instead of one per worker.
    first_fused: the first layer's backward kernel also runs the next forward product of that
    layer (label gemm_bwd_first), so gemm_fwd and gemm_bwd cover the layers above it."""
    n, b = w.n_workers, w.batch
    nw = 1 if shared_weights else n
    out = {}
    if w.model == "lsq":
        d = w.dims[0]
        out["lsq_steps"] = {"bytes": n * b * (d + 1) * 4, "flops": 4 * n * b * d}
        out["average"] = {"bytes": 8 * n * d, "flops": n * d}
        out["restart_mean"] = {"bytes": 4 * n * d + 4 * d, "flops": n * d}
        return out
    es = 2 if w.gemm_dtype == "bf16" else 4          # operand element size
    dims = w.dims
    layers = [(dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    m = sum(di * do + do for di, do in layers)
    pw = sum(di * do for di, do in layers)
    shadow = 2 if w.gemm_dtype == "bf16" else 0
    fwd_b = sum(nw * di * do * es + n * (b * di * es + b * do * es) for di, do in layers)
    fwd_f = sum(2 * n * b * di * do for di, do in layers)
    dx_b = sum(nw * di * do * es + n * (b * do * es + 2 * b * di * es) for di, do in layers[1:])
    dx_f = sum(2 * n * b * di * do for di, do in layers[1:])
    dw_b = sum(n * (di * do * (8 + shadow) + b * (di + do) * es) for di, do in layers)
    dw_f = fwd_f
    # fused backward kernel (bf16 operands): master read + write, shadow write, the activation and
    # delta panels, and the delta of the layer below; both products
    mom = 8 if getattr(w, "momentum", 0.0) != 0.0 else 0   # velocity read + write per element
    bwd_b = sum(n * (di * do * (10 + mom) + b * (di + do) * 2) for di, do in layers) + \
        sum(n * b * di * 2 for di, do in layers[1:])
    out["gemm_bwd"] = {"bytes": bwd_b, "flops": dw_f + dx_f}
    # first layer, backward + next forward in one pass: master read + write (the shadow is not
    # written), the minibatches of both iterations, the delta panel, the next activation; both
    # products
    d0, d1 = layers[0]
    first_b = n * (d0 * d1 * (8 + mom) + b * (2 * d0 + 2 * d1) * 2)
    first_f = 4 * n * b * d0 * d1
    out["gemm_bwd_first"] = {"bytes": first_b, "flops": first_f}
    if first_fused:
        l1_bwd_b = n * (d0 * d1 * (10 + mom) + b * (d0 + d1) * 2)
        l1_fwd_b = nw * d0 * d1 * es + n * (b * d0 * es + b * d1 * es)
        out["gemm_bwd"] = {"bytes": bwd_b - l1_bwd_b, "flops": dw_f + dx_f - 2 * n * b * d0 * d1}
        fwd_b, fwd_f = fwd_b - l1_fwd_b, fwd_f - 2 * n * b * d0 * d1
    out["gather"] = {"bytes": n * b * dims[0] * (4 + es), "flops": 0}
    out["gemm_fwd"] = {"bytes": fwd_b, "flops": fwd_f}
    out["gemm_dx"] = {"bytes": dx_b, "flops": dx_f}
    out["gemm_dw"] = {"bytes": dw_b, "flops": dw_f}
    # the loss-head launch also gathers the next iteration's minibatch (the stand-alone gather only
    # runs when no draw is waiting: the first iteration of a run)
    out["softmax_xent"] = {"bytes": n * b * dims[-1] * (4 + es) + out["gather"]["bytes"], "flops": 0}
    out["sgd_update"] = {"bytes": n * m * (12 + mom + shadow), "flops": (2 + (2 if mom else 0)) * n * m}
    # fused epoch kernel (one launch = `interval` iterations): per iteration the gathered rows and
    # all three products; the weights cross HBM once per launch (read + write), amortised here
    out["mlp2_epoch"] = {"bytes": n * b * (dims[0] + 1) * 4 + (8.0 + mom) * n * m / max(1, w.interval),
                         "flops": fwd_f + dx_f + dw_f}
    out["average"] = {"bytes": n * m * 8 + n * pw * shadow, "flops": n * m}
    # restart with the broadcast deferred: every replica read once, the node average (and its
    # bf16 image) written once
    out["restart_mean"] = {"bytes": n * m * 4 + m * 4 + pw * shadow, "flops": n * m}
    # I = 1, step and restart in one pass: the node average read and written once (+ bf16 image),
    # every worker's activation and delta panels read once; the weight-gradient product
    out["step_mean"] = {"bytes": m * 8 + pw * shadow + sum(n * b * (di + do) * 2 for di, do in layers),
                        "flops": dw_f}
    return out


def kernel_source_digest():
    """sha256 over the HIP sources: counter readings are only valid for the code they were taken on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1807_06629_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE
    readings (profiles/hbm_traffic.json), or None when there is no reading for this workload
    and kernel or the kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
    except Exception:
        return None
    rec = table.get(workload, {}).get(kernel)
    if not rec or rec.get("source_sha256") != kernel_source_digest():
        return None
    return rec.get("traffic_bytes_per_launch")


def measured_counters(workload, kernel):
    """Matrix-core busy fraction, LDS bank-conflict share and wave occupancy of `kernel` from the
    committed rocprofv3 --pmc readings (same table and validity rule as measured_traffic)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
    except Exception:
        return None
    rec = table.get(workload, {}).get(kernel)
    if not rec or rec.get("source_sha256") != kernel_source_digest():
        return None
    return rec.get("counters")


def cpu_baseline(w, inp, budget_s=15.0):
    """The oracle as it stands, timed on the host cores on a bounded number of iterations:
    once with the BLAS threads numpy starts by itself (all-core figure, `value`) and once
    restricted to one thread (`single_thread`), the latter on worker 0's share of an iteration
    when a whole iteration would not fit the budget (workers are independent inside an
    iteration, so samples/s scales with the share)."""
    import oracle
    from threadpoolctl import threadpool_info, threadpool_limits
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    common = dict(model=w.model, dims=w.dims, activation=w.activation, x0=inp["x0"], batch=w.batch,
                  lr=w.lr, interval=w.interval, seed=w.index_seed, bf16=(w.gemm_dtype == "bf16"),
                  momentum=w.momentum, momentum_restart=w.momentum_restart)
    full = dict(common, features=inp["features"], targets=inp["targets"], n_workers=w.n_workers)
    one = dict(common, features=inp["features"][:1], targets=inp["targets"][:1], n_workers=1)

    def timed(args, iters):
        t0 = time.perf_counter()
        oracle.run_prsgd(iterations=iters, **args)
        return time.perf_counter() - t0

    def sample(args, n_workers, what):
        t_one = timed(args, 1)                      # also warms the allocator and the BLAS threads
        iters = int(max(1, min(w.iterations, budget_s / max(t_one, 1e-6))))
        dt = timed(args, iters)
        restarts = iters // w.interval
        note = "%d iterations of %s (incl. %d restart averages), %.1f s, numpy float64" % (
            iters, what, restarts, dt)
        if iters < 2 * w.interval:
            note += "; shorter than two restart intervals: the rate is extrapolated linearly in T " \
                    "(a restart average is one pass over N*m doubles, far below one iteration's cost)"
        return n_workers * w.batch * iters / dt, note, t_one

    value, note, t_one = sample(full, w.n_workers, "workload %s" % w.name)
    out = {"value": value, "unit": "samples/s", "cores": int(cores), "kind": "oracle", "sample": note}
    with threadpool_limits(limits=1):
        if t_one * cores <= 2 * budget_s:           # a whole single-threaded iteration fits
            v1, n1, _ = sample(full, w.n_workers, "workload %s" % w.name)
        else:
            v1, n1, _ = sample(one, 1, "worker 0's share (1/%d) of workload %s" % (w.n_workers, w.name))
    out["single_thread"] = {"value": v1, "unit": "samples/s", "cores": 1, "sample": n1}
    return out


def restart_average_at_hbm_scale(prsgd, drivers, get_workload, make_inputs, reps=20):
    """The restart kernels (eq. 2) timed on a replica set far larger than the caches: the
    largest workload's replicas ([8][54.4M] fp32 + bf16 shadow) with a token data shard, in the
    alternation they run in (one local iteration, then the restart).  `average` = read every
    replica, overwrite every replica (4.36 GB per pass); `restart_mean` = the deferred-broadcast
    form, every replica read, the average written once (2.07 GB).  HIP events on the library's
    stream, through the library's own profiling."""
    w = get_workload("c5").scaled(rows_per_worker=64, batch=8)
    h = drivers.open_workload(w, make_inputs(w), device="cuda:0")
    out = {"workload": "replica set of c5: N=8, m=54440936, fp32 master + bf16 shadow; "
                       "one local iteration (B=8) between restarts"}
    for lazy, label in ((False, "average"), (True, "restart_mean")):
        prsgd.prsgd_set_lazy_restart(h, lazy)
        def once():
            prsgd.prsgd_local_steps(h, 1)
            prsgd.prsgd_average(h)
        for _ in range(3):
            once()
        prsgd.prsgd_profile_enable(h, True)
        for _ in range(reps):
            once()
        stats = {s["name"]: s for s in prsgd.prsgd_profile_read(h)}
        prsgd.prsgd_profile_enable(h, False)
        work = algorithmic_work(w)[label]["bytes"]
        sec = stats[label]["total_ms"] * 1e-3 / stats[label]["launches"]
        out[label] = {"bytes": work, "avg_us": 1e6 * sec, "GBps": work / sec / 1e9,
                      "frac_of_hbm_peak": work / sec / 1e9 / HBM_PEAK_GBPS,
                      "launches_timed": stats[label]["launches"]}
    prsgd.prsgd_destroy(h)
    return out


def standalone_update_at_hbm_scale(prsgd, n_elems=1 << 28, reps=20):
    """The stand-alone elementwise form of eq. (3), x <- x - gamma g (+ bf16 image of x), on
    2^28 elements (1 GiB per fp32 vector): 12 B/element of fp32 traffic + 2 B/element shadow."""
    import torch
    x = torch.zeros(n_elems, dtype=torch.float32, device="cuda:0")
    g = torch.ones(n_elems, dtype=torch.float32, device="cuda:0")
    sh = torch.zeros(n_elems, dtype=torch.bfloat16, device="cuda:0")
    out = {}
    for label, shadow, bpe in (("fp32", None, 12), ("fp32_with_bf16_shadow", sh, 14)):
        for _ in range(3):
            prsgd.prsgd_sgd_update(x, g, 1e-3, shadow=shadow)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            prsgd.prsgd_sgd_update(x, g, 1e-3, shadow=shadow)
        stop.record()
        torch.cuda.synchronize()
        sec = start.elapsed_time(stop) * 1e-3 / reps
        out[label] = {"bytes": bpe * n_elems, "avg_us": 1e6 * sec, "GBps": bpe * n_elems / sec / 1e9,
                      "frac_of_hbm_peak": bpe * n_elems / sec / 1e9 / HBM_PEAK_GBPS}
    out["symbol"] = "update_kernel"
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--interval", type=int, default=None)
    ap.add_argument("--unfused", action="store_true", help="separate elementwise update kernel")
    ap.add_argument("--eager-restart", action="store_true",
                    help="restart with the averaging kernel that overwrites every replica at once")
    ap.add_argument("--separate-first-layer", action="store_true",
                    help="first layer: backward kernel and next forward product as two launches")
    ap.add_argument("--momentum", type=float, default=None,
                    help="momentum of the local steps (default: the workload's, 0 = eq. 3 as printed)")
    ap.add_argument("--momentum-restart", choices=["keep", "average", "reset"], default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-average", action="store_true",
                    help="skip the extra HBM-scale timing of the averaging kernel")
    ap.add_argument("--rows", type=int, default=None, help="rows per worker (default: workload's)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="time the plain copy kernel (known traffic) instead of a workload")
    ap.add_argument("--copy-mib", type=int, default=1024)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (the N workers are simulated on it); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    if not os.path.exists(os.path.join(ROOT, "paper_1807_06629_amd", "libprsgd.so")):
        from paper_1807_06629_amd.build import build
        build()
    from paper_1807_06629_amd import drivers, prsgd
    from workloads import get_workload, make_inputs

    if args.calibrate_copy:
        n_bytes = args.copy_mib << 20
        src = torch.ones(n_bytes // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        reps = args.steps if args.steps is not None else 20
        for _ in range(3):
            prsgd.prsgd_copy_bytes(dst, src)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            prsgd.prsgd_copy_bytes(dst, src)
        stop.record()
        torch.cuda.synchronize()
        ms = start.elapsed_time(stop) / reps
        print(json.dumps({"kernel": "copy_kernel", "bytes_read": n_bytes, "bytes_written": n_bytes,
                          "launches": reps + 3, "avg_us": 1e3 * ms,
                          "GBps": 2 * n_bytes / (ms * 1e-3) / 1e9,
                          "frac_of_hbm_peak": 2 * n_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}))
        return 0

    w = get_workload(args.workload)
    if args.interval is not None:
        w = w.scaled(interval=args.interval)
    if args.rows is not None:
        w = w.scaled(rows_per_worker=args.rows)
    if args.momentum is not None:
        w = w.scaled(momentum=args.momentum)
    if args.momentum_restart is not None:
        w = w.scaled(momentum_restart=args.momentum_restart)
    steps = args.steps if args.steps is not None else min(w.iterations, 2000)
    warmup = args.warmup if args.warmup is not None else min(2 * w.interval, 32)

    inp = make_inputs(w)
    stream = torch.cuda.Stream(device="cuda:0")
    with torch.cuda.stream(stream):
        h = drivers.open_workload(w, inp, device="cuda:0", fused_update=not args.unfused,
                                  stream=stream)
    if args.eager_restart:
        prsgd.prsgd_set_lazy_restart(h, False)
    if args.separate_first_layer:
        prsgd.prsgd_set_first_layer_fusion(h, False)
    torch.cuda.synchronize()

    prsgd.prsgd_run(h, warmup, w.interval)
    prsgd.prsgd_set_iteration(h, 0)                  # timed region starts on an epoch boundary
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    prsgd.prsgd_run(h, steps, w.interval)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prsgd.prsgd_status(h)                            # raises if any launch of the run gave up
    loss = float(prsgd.prsgd_read_loss(h).mean())

    # per-kernel durations: the same steps again with every launch bracketed by HIP events on
    # the library's stream
    # whole restart intervals, so that every launch of an epoch kernel covers `interval`
    # iterations like the launches the traffic counters were read on
    prof_steps = w.interval * max(2, -(-32 // w.interval))
    prsgd.prsgd_set_iteration(h, 0)
    prsgd.prsgd_profile_enable(h, True)
    prsgd.prsgd_run(h, prof_steps, w.interval)
    stats = prsgd.prsgd_profile_read(h)
    prsgd.prsgd_profile_enable(h, False)

    one_pass = (w.interval == 1 and w.model == "mlp" and w.gemm_dtype == "bf16" and not args.unfused
                and not args.eager_restart and w.momentum == 0.0 and w.batch <= 128)
    first_fused = any(s["name"] == "gemm_bwd_first" for s in stats)
    work = algorithmic_work(w, shared_weights=one_pass, first_fused=first_fused)
    prof_key = w.name + ("_I1" if one_pass else "")      # counter readings are kept per launch pattern
    kernels = {}
    # the work table is per iteration; kernels launched once per layer are priced per launch (they do
    # not run in every iteration: the pass that closes an epoch replaces the per-replica backward
    # kernels by backward-data products and the stacked weight-gradient product)
    n_layers = len(w.dims) - 1
    per_iteration_launches = {"gemm_fwd": n_layers - (1 if first_fused else 0),
                              "gemm_bwd": n_layers - (1 if first_fused else 0),
                              "gemm_dx": n_layers - 1, "gemm_dw": n_layers, "step_mean": n_layers}
    for s in stats:
        per_iter = work.get(s["name"], {"bytes": 0, "flops": 0})
        calls = prof_steps if s["name"] not in ("average", "restart_mean") else max(1, prof_steps // w.interval)
        if s["name"] in ("lsq_steps", "mlp2_epoch"):
            calls = prof_steps                        # one launch covers several iterations
        if s["name"] in ("gather", "gemm_bwd_first", "softmax_xent", "sgd_update"):
            calls = s["launches"]                     # one launch per iteration in which they run
        if s["name"] in per_iteration_launches and w.model == "mlp":
            calls = s["launches"] / max(1, per_iteration_launches[s["name"]])
        tot_bytes, tot_flops = per_iter["bytes"] * calls, per_iter["flops"] * calls
        sec = s["total_ms"] * 1e-3
        kernels[s["name"]] = {
            "launches": s["launches"], "avg_us": 1e3 * s["total_ms"] / s["launches"],
            "total_ms": s["total_ms"], "GBps": tot_bytes / sec / 1e9 if sec > 0 else None,
            "TFLOPs": tot_flops / sec / 1e12 if sec > 0 else None,
            "bytes_per_launch": tot_bytes / s["launches"], "flops_per_launch": tot_flops / s["launches"],
        }
    dom = max(kernels, key=lambda k: kernels[k]["total_ms"])
    kd = kernels[dom]
    peak_tf = MFMA_PEAK_TFLOPS[w.gemm_dtype if w.model == "mlp" else "f32"]
    t_hbm = kd["bytes_per_launch"] / (HBM_PEAK_GBPS * 1e9)
    t_mfma = kd["flops_per_launch"] / (peak_tf * 1e12)
    if t_hbm >= t_mfma:
        roof = {"bound": "hbm", "achieved": kd["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": kd["GBps"] / HBM_PEAK_GBPS}
    else:
        roof = {"bound": "mfma", "achieved": kd["TFLOPs"], "peak": peak_tf, "unit": "TFLOP/s",
                "frac": kd["TFLOPs"] / peak_tf}
    # matrix-core view of the same kernel: flops / time against the chip's peak, beside the most
    # the kernel's arithmetic intensity allows at the HBM peak (the products here are skinny:
    # every replica has private weights and at most 128 minibatch rows)
    if kd["flops_per_launch"] > 0 and kd["bytes_per_launch"] > 0:
        ai = kd["flops_per_launch"] / kd["bytes_per_launch"]
        roof["mfma"] = {"achieved_TFLOPs": kd["TFLOPs"], "peak_TFLOPs": peak_tf,
                        "frac_of_peak": kd["TFLOPs"] / peak_tf,
                        "flop_per_byte": ai,
                        "ceiling_frac_at_hbm_peak": min(1.0, ai * HBM_PEAK_GBPS * 1e9 / (peak_tf * 1e12)),
                        "busy_counters": measured_counters(prof_key, dom)}
    roof.update({"traffic": measured_traffic(prof_key, dom), "kernel": dom, "symbol": KERNEL_SYMBOL.get(dom, dom),
                 "avg_launch_us": kd["avg_us"], "launches_timed": kd["launches"],
                 "algorithmic_bytes_per_launch": kd["bytes_per_launch"],
                 "algorithmic_flops_per_launch": kd["flops_per_launch"]})

    restart = None
    for label in ("restart_mean", "average"):
        avg = kernels.get(label)
        if avg:
            restart = {"kernel": label, "symbol": KERNEL_SYMBOL[label], "GBps": avg["GBps"],
                       "frac_of_hbm_peak": avg["GBps"] / HBM_PEAK_GBPS, "avg_us": avg["avg_us"],
                       "bytes": avg["bytes_per_launch"]}
            break

    out = {
        "metric": "samples/sec across N replicas at interval I; restart-average HBM GB/s",
        "value": w.n_workers * w.batch * steps / wall,
        "unit": "samples/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * wall / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if (w.model == "mlp" and w.gemm_dtype == "bf16") else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %s %s N=%d B=%d I=%d n=%d lr=%g %s" % (
            w.name, w.model, "-".join(str(d) for d in w.dims), w.n_workers, w.batch, w.interval,
            w.rows_per_worker, w.lr, w.activation),
            "n_workers": w.n_workers, "batch": w.batch, "interval": w.interval,
            "fused_update": not args.unfused, "deferred_broadcast": not args.eager_restart,
            "momentum": w.momentum, "momentum_restart": w.momentum_restart,
            "last_minibatch_loss": loss},
        "roofline": roof,
        "restart_average": restart,
        "kernels": {k: {"avg_us": round(v["avg_us"], 3), "launches": v["launches"],
                        "GBps": v["GBps"], "TFLOPs": v["TFLOPs"]} for k, v in kernels.items()},
    }
    prsgd.prsgd_destroy(h)
    del h
    torch.cuda.empty_cache()
    if not args.no_hbm_average:
        # the second half of the metric, whatever the workload: both restart kernels and the
        # stand-alone update on a replica set far larger than the caches
        out["restart_average_hbm"] = restart_average_at_hbm_scale(prsgd, drivers, get_workload,
                                                                  make_inputs)
        out["sgd_update_hbm"] = standalone_update_at_hbm_scale(prsgd)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
