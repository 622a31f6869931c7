#!/usr/bin/env python3
"""Benchmark of the subsampled Gauss-Newton path on one MI355X.

One step = one pass of the whole path on a synthetic workload already resident in HBM:
dn_forward (f), dn_grad, dn_jacobian_prep, `mv_reps` x dn_gn_matvec (full), `mv_reps` x
dn_gn_matvec (per-layer block-diagonal), dn_cg (full) and dn_cg (block-diagonal) with the
configuration's CG iteration count.  Prints ONE JSON line:

  value        Gauss-Newton matvecs/s = full products per second inside the timed steps
               (HIP events around the `mv_reps` back-to-back full products of every step)
  ms_per_step  wall time of the whole step
  roofline     the dominant kernel of dn_gn_matvec: algorithmic flops (or bytes) per launch over
               its mean duration, measured with HIP events in a second pass of the same steps
  cpu_baseline the fp64 oracle's product rate on the host cores, on the same workload

  extras       (--extras only, measured after the timed steps) partition-mode product and CG, the product
               without stored blocks, and whole Newton iterations

  per_config   the other configurations (2, 3, 4 by default), short protocol, same quantities

The timed steps carry no instrumentation inside the library; the event brackets around the dominant kernel
come from a second pass of the same steps.

python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--per-config 2,3,4|none] [--extras]
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

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E


def work_per_launch(cfg, s):
    """Algorithmic work of one launch of each product kernel class (Section 4.2 / Section 5.2 costs).

    GEMM classes: 2 flops per multiply-add of the |T_{m-1}| x |T_m| term summed over layers.
    Streaming classes: bytes of the stored blocks that one launch must read once.
    """
    d = cfg.dims
    L = len(d) - 1
    wsum = sum(d[m - 1] * d[m] for m in range(1, L + 1))
    hid = sum(d[m] for m in range(1, L))
    pbytes = 4.0 * s * d[L] * hid
    # the two-pass kernels stream the blocks of layers 1..L-2 only (block L-1 is applied as a dense product)
    pbytes_streamed = 4.0 * s * d[L] * sum(d[m] for m in range(1, L - 1))
    return {
        "gemm_q_matvec": ("mfma", 2.0 * s * wsum),
        "gemm_tn_matvec": ("mfma", 2.0 * s * wsum),
        "jv_jtv_fused": ("hbm", pbytes),
        "jv_jtv_band": ("hbm", pbytes_streamed),
        "jv_rows": ("hbm", pbytes_streamed),
        "jtv_cols": ("hbm", pbytes_streamed),
        "tn_reduce": ("hbm", 4.0 * 3 * cfg.n_params),
    }


def measured_traffic(workload, kernel_class):
    """HBM bytes per launch (fetch + write) of a kernel class from the committed counter summary, or None.

    The summary is written from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this same script and
    scaled by what the same counters read for a plain copy kernel of known size.
    """
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == kernel_class:
                    return float(parts[1]) + float(parts[2])
    except OSError:
        pass
    return None


def matvec_flops(cfg, s):
    d = cfg.dims
    L = len(d) - 1
    return s * (4.0 * sum(d[m - 1] * d[m] for m in range(1, L + 1)) + 4.0 * d[L] * sum(d[m] for m in range(1, L)))


def cpu_baseline(cfg, X, theta, S, budget_s=20.0):
    """Time the oracle's full product on the host, on a bounded sample of the workload.

    The oracle's product is a sum over the samples of S, so its cost is proportional to the number of samples:
    a pilot on a few samples sizes a sample of about `budget_s` seconds of work (all of S where that fits), and
    the rate is scaled to whole products over |S| samples.
    """
    import numpy as np
    from oracle import dn_oracle as orc
    import dn_inputs
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    th = theta.astype(np.float64)
    v = dn_inputs.make_probe(cfg, 0).astype(np.float64)
    s_all = int(S.shape[0])
    pilot = min(s_all, 64)
    XP = X[S[:pilot]].astype(np.float64)
    orc.gn_matvec(th, cfg.dims, cfg.C, XP, v)      # warm-up (BLAS thread start-up)
    t0 = time.perf_counter()
    orc.gn_matvec(th, cfg.dims, cfg.C, XP, v)
    per_sample = (time.perf_counter() - t0) / pilot
    if per_sample * s_all <= budget_s:
        rows, reps_max = s_all, 20
    else:
        rows, reps_max = max(pilot, min(s_all, int(budget_s / per_sample))), 1
    XS = X[S[:rows]].astype(np.float64)
    t0 = time.perf_counter()
    reps = 0
    while True:
        orc.gn_matvec(th, cfg.dims, cfg.C, XS, v)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= reps_max:
            break
    products = reps * rows / s_all            # whole products' worth of work done
    sample = (f"{reps} full G^S v products" if rows == s_all else
              f"{reps} product over the first {rows} of the |S|={s_all} samples, rate scaled by {rows}/{s_all}")
    return {"value": products / el, "unit": "matvecs/s", "cores": int(threads), "kind": "oracle",
            "seconds": el, "sample": sample + ", same theta/X_S/v as the GPU run, numpy fp64"}


def run_config(args, index, steps, warmup, with_cpu_baseline, extras):
    """All measurements of one configuration; returns the result dictionary (the JSON line's fields)."""
    import numpy as np
    import torch
    import dn_inputs
    import paper_1802_00130_amd as dn

    cfg = dn_inputs.config(index)
    dev = torch.device("cuda:0")
    X = dn_inputs.make_X(cfg)
    Y = dn_inputs.make_Y(cfg)
    theta = dn_inputs.make_theta(cfg)
    S = dn_inputs.make_subset(cfg)
    v = dn_inputs.make_probe(cfg, 0)
    dX, dY = torch.from_numpy(X).to(dev), torch.from_numpy(Y).to(dev)
    del Y
    dtheta, dS, dv = torch.from_numpy(theta).to(dev), torch.from_numpy(S).to(dev), torch.from_numpy(v).to(dev)
    ctx = dn.Context(cfg.dims, cfg.C, cfg.l, cfg.s)
    n = ctx.n
    g = torch.empty(n, dtype=torch.float32, device=dev)
    out = torch.empty(n, dtype=torch.float32, device=dev)
    d = torch.empty(n, dtype=torch.float32, device=dev)
    R = args.mv_reps

    phases = ["forward", "grad", "jacobian_prep", "matvec_full", "matvec_blockdiag", "cg_full", "cg_blockdiag"]

    def step(ev=None):
        def mark(k):
            if ev is not None:
                ev[k].record()
        mark(0)
        dn.dn_forward(ctx, dtheta, dX, dY)
        mark(1)
        dn.dn_grad(ctx, dtheta, dX, dY, g, want_f=False)
        mark(2)
        dn.dn_jacobian_prep(ctx, dtheta, dX, dS)
        mark(3)
        for _ in range(R):
            dn.dn_gn_matvec(ctx, dv, out, dn.DN_FULL)
        mark(4)
        for _ in range(R):
            dn.dn_gn_matvec(ctx, dv, out, dn.DN_BLOCKDIAG)
        mark(5)
        dn.dn_cg(ctx, g, cfg.lam, 0.0, cfg.cg_iters, dn.DN_FULL, d)
        mark(6)
        dn.dn_cg(ctx, g, cfg.lam, 0.0, cfg.cg_iters, dn.DN_BLOCKDIAG, d)
        mark(7)

    if args.copy_calib and cfg.L >= 2:
        dn.dn_jacobian_prep(ctx, dtheta, dX, dS)
        Pc = torch.empty(cfg.s * cfg.dims[-1] * cfg.dims[1], dtype=torch.float32, device=dev)
        dn.dn_jacobian_read(ctx, 1, Pc)     # unpad_rows_kernel: reads and writes 4*|S|*n_L*n_1 bytes
        torch.cuda.synchronize()
        print(f"copy-calib: unpad_rows_kernel moved {4 * Pc.numel()} bytes each way", file=sys.stderr)
        del Pc

    # warm-up, with every kernel class bracketed, to find the dominant product kernel
    work = work_per_launch(cfg, cfg.s)
    ctx.profile_select(None)
    ctx.profile_enable(True)
    ctx.profile_reset()
    for _ in range(max(1, warmup)):
        step()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    warm_kernel_ms = {k: (ms / cnt if cnt else 0.0) for k, (ms, cnt) in prof.items() if cnt}
    dominant = max(work, key=lambda k: prof.get(k, (0.0, 0))[0])
    ctx.profile_enable(False)

    # timed region: no instrumentation inside the library, only the phase marks of the step
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    status = ctx.sync_status()
    if status != 0:
        raise RuntimeError(f"bench.py: the library reported status {status} after the timed steps")

    # second pass, outside `value`: the same steps with the dominant kernel class bracketed by HIP events on
    # the library's stream
    ctx.profile_select([dominant])
    ctx.profile_enable(True)
    ctx.profile_reset()
    for _ in range(max(1, min(steps, args.profile_steps))):
        step()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    band_phases = None
    if dominant == "jv_jtv_band":
        # where a work-group of that kernel spends its time: one more full product with the kernel's phase clocks on
        ctx.profile_band_phases(True)
        dn.dn_gn_matvec(ctx, dv, out, dn.DN_FULL)
        band_phases = ctx.profile_band_read()
        ctx.profile_band_phases(False)

    # what an EMPTY event bracket reads on this stream while it is busy: the part of avg_kernel_ms that is
    # not kernel time (a profiler's per-dispatch duration does not contain it)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(8)]
    for a, b in pairs:
        dn.dn_gn_matvec(ctx, dv, out, dn.DN_FULL)
        a.record()
        b.record()
    torch.cuda.synchronize()
    bracket_ms = sum(a.elapsed_time(b) for a, b in pairs) / len(pairs)

    ex = None
    if extras:
        def timed(fn, reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn()
            torch.cuda.synchronize()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        # split structure 1-2-...-2-1: every hidden layer in two groups (Section 3.1), as in the paper's runs
        split = tuple(1 if m in (0, cfg.L) else 2 for m in range(cfg.L + 1))
        nparts = ctx.set_split(split)
        ex = {"split": "-".join(map(str, split)), "partitions": nparts}
        ex["matvec_partition_ms"] = timed(lambda: dn.dn_gn_matvec(ctx, dv, out, dn.DN_PARTITION), R)
        ex["cg_partition_ms_per_iteration"] = timed(
            lambda: dn.dn_cg(ctx, g, cfg.lam, 0.0, cfg.cg_iters, dn.DN_PARTITION, d), 1) / cfg.cg_iters
        ex["matvec_rop_ms"] = timed(lambda: dn.dn_gn_matvec_rop(ctx, dv, out), R)
        # outer iterations (Section 4.5) from the initial point: lambda carried over, forward pass of the
        # accepted line-search point reused by the next gradient
        th, dprev, lam = dtheta.clone(), torch.zeros_like(dtheta), cfg.lam
        iters, cg_total = 4, 0
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for k in range(iters):
            st = dn.dn_newton_step(ctx, th, dX, dY, dS, dprev, lam, cfg.cg_iters, reuse_forward=(k > 0))
            lam = st["lam"]
            cg_total += st["cg_iters"]
        torch.cuda.synchronize()
        ex["newton_ms_per_iteration"] = (time.perf_counter() - t1) * 1000.0 / iters
        ex["newton_cg_iterations"] = cg_total / iters
        ex["newton_f_last"] = st["f_new"]

    phase_ms = {p: 0.0 for p in phases}
    for evs in events:
        for i, p in enumerate(phases):
            phase_ms[p] += evs[i].elapsed_time(evs[i + 1])
    for p in phases:
        phase_ms[p] /= steps
    mv_ms = phase_ms["matvec_full"] / R
    value = 1000.0 / mv_ms
    ms_per_step = wall * 1000.0 / steps

    bound, unit_work = work[dominant]
    tot_ms, launches = prof[dominant]
    avg_ms = tot_ms / max(1, launches)
    if bound == "mfma":
        achieved = unit_work / (avg_ms * 1e-3) / 1e12
        peak, unit = PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"
    else:
        achieved = unit_work / (avg_ms * 1e-3) / 1e9
        peak, unit = PEAK_HBM_GBS, "GB/s"
    roofline = {"bound": bound, "kernel": dominant, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": measured_traffic(cfg.name, dominant), "avg_kernel_ms": avg_ms,
                "launches": int(launches), "work_per_launch": unit_work, "empty_event_bracket_ms": bracket_ms}
    if band_phases is not None:
        roofline["band_phase_cycles"] = band_phases

    mv_tflops = matvec_flops(cfg, cfg.s) / (mv_ms * 1e-3) / 1e12
    res = {
        "metric": "Gauss-Newton matvecs/sec and achieved fp32-MFMA TFLOP/s, 1xMI355X",
        "value": value, "unit": "matvecs/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "dims": list(cfg.dims), "l": cfg.l, "subsample": cfg.s, "C": cfg.C,
                   "lambda": cfg.lam, "cg_iters": cfg.cg_iters, "mv_reps": R, "seed": cfg.seed},
        "matvec_ms": mv_ms, "matvec_blockdiag_ms": phase_ms["matvec_blockdiag"] / R,
        "matvec_tflops": mv_tflops, "matvec_frac_of_fp32_mfma_peak": mv_tflops / PEAK_FP32_MFMA_TFLOPS,
        "cg_ms_per_iteration": phase_ms["cg_full"] / cfg.cg_iters,
        "phase_ms": phase_ms,
        "warmup_avg_kernel_ms": warm_kernel_ms,
        "roofline": roofline,
    }
    if ex is not None:
        res["extras"] = ex
    ctx.close()
    del ctx, dX, dY, g, out, d
    torch.cuda.empty_cache()
    if with_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, X, theta, S)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5,
                    help="BASELINE configuration 1..5 (default 5: the largest, on which the metric is quoted)")
    ap.add_argument("--mv-reps", type=int, default=20)
    ap.add_argument("--profile-steps", type=int, default=2,
                    help="steps of the second, untimed pass in which the dominant kernel is bracketed by events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-config", type=str, default=None,
                    help="comma-separated further configurations measured after the headline one with a short "
                         "protocol (3 steps) into a \"per_config\" object; default 2,3,4 when --config is 5, "
                         "\"none\" to skip")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run one plain copy kernel of known size (dense copy of stored block P^1) so that "
                         "a counter run can be scaled by what the same counter reads for that copy")
    ap.add_argument("--extras", action="store_true",
                    help="after the timed steps also time the rows beyond the headline path (partition-mode product "
                         "and CG, product without stored blocks, whole Newton iterations) into an \"extras\" object")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    res = run_config(args, args.config, args.steps, args.warmup, not args.no_cpu_baseline, args.extras)
    others = args.per_config
    if others is None:
        others = "2,3,4" if args.config == 5 else "none"
    if others != "none":
        keep = ("matvec_ms", "matvec_blockdiag_ms", "matvec_tflops", "matvec_frac_of_fp32_mfma_peak",
                "cg_ms_per_iteration", "ms_per_step", "steps", "warmup", "phase_ms", "roofline")
        res["per_config"] = {}
        for k in (int(x) for x in others.split(",")):
            r = run_config(args, k, 3, 1, False, False)
            res["per_config"][r["config"]["workload"]] = {key: r[key] for key in keep}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
