#!/usr/bin/env python3
"""Benchmark of the stencil hot path on one MI355X.

One "step" = one pass of the stencil over the workload's matrix (all of its iterations) at
the workgroup size the sweep found best.  Before the timed region the script runs the sweep
of Section 5 over the workload's whole size list (every size: 3 warm-ups + `--reps` samples),
reduces it (best size, speedup over the fixed sizes 4x4 and 32x4 / 4x32, best/worst) and asks
the predictor for a size.  Inputs are generated on the host from a seed and are resident in
HBM before anything is timed.

Prints ONE JSON line.  `value` = Gcells/s (cell updates per second) of the timed steps;
`roofline` prices the stencil kernel's algorithmic bytes (one read + one write per cell
update) over its HIP-event-measured launch time against the 8 TB/s HBM peak; `cpu_baseline`
is the CPU oracle timed on a bounded sample of the same workload on the host cores.
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
FP32_VECTOR_PEAK_TFLOPS = 157.3      # published: packed fp32 fma on 256 CUs x 4 SIMDs x 16 lanes at 2.4 GHz


def flops_per_cell_update(w):
    """fp32 operations the customising function states per cell and application (None: integer)."""
    n, s_, e, w_ = w.halo
    taps = (n + s_ + 1) * (e + w_ + 1)
    if w.kernel == "heat":
        return 7                     # three adds, 4u, the subtraction, alpha * t, the final add
    if w.kernel == "weighted_sum":
        return 2 * taps - 1 if w.dtype == "f32" else None
    if w.kernel == "sincos":
        return 3 * taps + 1          # per cell of the region: w * sin + cos and the running sum; sin and cos once
    return None

# mappings swept besides the paper's one element per work-item with a local-memory tile:
# (staging, cells_rows, cells_cols)
# ... or ("temporal", cells_rows, 4, applications per launch) for the iterated heat workload
MAPPINGS = {
    "weighted_sum": [("local", 1, 1), ("local", 2, 4), ("local", 4, 4), ("direct", 1, 4), ("direct", 2, 4),
                     ("direct", 4, 4), ("stream", 5, 4), ("stream", 10, 4), ("stream", 20, 4)],
    "heat": [("local", 1, 1), ("local", 2, 4), ("local", 4, 4), ("direct", 1, 4), ("direct", 2, 4),
             ("temporal", 2, 4, 2), ("temporal", 4, 4, 2), ("temporal", 4, 4, 3), ("temporal", 2, 4, 4),
             ("temporal", 4, 4, 4), ("temporal", 8, 4, 4),
             ("stream", 16, 4, 4), ("stream", 36, 4, 4), ("stream", 40, 4, 6), ("stream", 38, 4, 8),
             ("stream", 74, 4, 8)],
    "sincos": [("local", 1, 1), ("local", 2, 4), ("local", 4, 4), ("local", 8, 4),
               ("stream", 64, 4), ("stream", 67, 4), ("stream", 89, 4), ("stream", 134, 4)],
    "life": [("local", 1, 1), ("local", 1, 16), ("local", 2, 16), ("direct", 1, 16), ("direct", 2, 16),
             ("direct", 4, 16), ("temporal", 2, 16, 2), ("temporal", 4, 16, 2), ("temporal", 2, 16, 4), ("temporal", 4, 16, 4),
             ("temporal", 8, 16, 4), ("stream", 16, 4, 4), ("stream", 40, 4, 6), ("stream", 40, 4, 8),
             ("stream", 20, 8, 8)],
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = per-workload default)")
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--reps", type=int, default=30, help="timed samples per workgroup size in the sweep")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-predictor", action="store_true", help="skip the leave-one-out predictor study")
    ap.add_argument("--quick", action="store_true", help="sweep a thinned size list (development only)")
    ap.add_argument("--wg", default="", help="R,C: skip the sweep and time this workgroup size (profiling runs)")
    ap.add_argument("--mapping", default="", help="staging,cells_rows,cells_cols to go with --wg, e.g. direct,2,4")
    ap.add_argument("--nt-store", default=None, choices=["0", "1"],
                    help="force plain (0) or non-temporal (1) output stores instead of timing both")
    ap.add_argument("--copy-only", action="store_true",
                    help="launch only the plain copy kernel on the workload's matrix (counter calibration)")
    return ap.parse_args()


def sweep_summary(res, cells_per_sample):
    import math as m
    legal = res.legal()
    out = {
        "sizes": len(res.sizes),
        "refused": sum(1 for s in res.status if s != 0),
        "best_wg": list(res.best) if res.best else None,
        "best_ms": res.best_ms,
        "best_gcells_s": cells_per_sample / res.best_ms / 1e6 if res.best else None,
        "worst_ms": res.worst_ms,
        "best_over_worst": res.worst_ms / res.best_ms if res.best else None,
    }
    for name, wg in (("4x4", (4, 4)), ("32x4", (32, 4)), ("4x32", (4, 32))):
        t = res.ms_of(wg)
        out["speedup_over_" + name] = (t / res.best_ms) if (res.best and not m.isnan(t)) else None
        out["gcells_s_" + name] = (cells_per_sample / t / 1e6) if not m.isnan(t) else None
    return out, legal


def apply_mapping(st, mapping):
    st.set_mapping(*mapping[:3])
    if len(mapping) > 3:
        st.set_option(1, mapping[3])      # STENCIL_OPT_TEMPORAL_DEPTH


def mapping_name(mapping):
    return "%s %dx%d" % tuple(mapping[:3]) + (" depth %d" % mapping[3] if len(mapping) > 3 else "")


def sweep_burst(w):
    """Applications per timed sample.  An event pair costs a few microseconds, so a sample is
    a burst of back-to-back applications long enough (>= ~100 us at a nominal 4 TB/s) to make
    that negligible; at least 10 for the iterated workloads."""
    est_us = w.rows * w.cols * w.bytes_per_cell_update / 4e12 * 1e6
    burst = int(min(20, max(1, math.ceil(100.0 / max(est_us, 1e-3)))))
    return max(burst, 24) if w.iters > 1 else burst      # 24: a multiple of every temporal depth swept


# the vectorised mapping each kernel is usually fastest with (predictor study)
FAST_MAPPING = {"weighted_sum": ("local", 2, 4), "heat": ("direct", 2, 4), "sincos": ("local", 2, 4),
                "life": ("direct", 2, 16)}


# strong configurations of each kernel, swept together (stencil_sweep_configs) for the per-workload
# figures of the workloads that are not the one being benchmarked:
# (staging, cells_rows, cells_cols, applications per launch or 0, workgroup size)
STRONG_CONFIGS = {
    "weighted_sum": [("local", 2, 4, 0, (16, 8)), ("local", 2, 4, 0, (8, 8)), ("direct", 2, 4, 0, (8, 16)),
                     ("direct", 4, 4, 0, (4, 128)), ("local", 4, 4, 0, (16, 8)), ("stream", 10, 4, 0, (1, 64)),
                     # the same with non-temporal output stores (numbering as is)
                     ("local", 2, 4, 0, (16, 8), -1, 1), ("direct", 2, 4, 0, (8, 16), -1, 1),
                     ("stream", 10, 4, 0, (1, 64), -1, 1), ("stream", 5, 4, 0, (1, 64), -1, 1)],
    "life": [("direct", 2, 16, 0, (2, 128)), ("direct", 4, 16, 0, (1, 256)), ("temporal", 2, 16, 4, (64, 8)), ("stream", 40, 4, 8, (1, 64)),
             ("stream", 40, 4, 8, (4, 64)), ("stream", 40, 4, 6, (1, 64))],
    "heat": [("direct", 2, 4, 0, (4, 16)), ("temporal", 2, 4, 4, (32, 32)), ("stream", 38, 4, 8, (1, 64)),
             ("stream", 38, 4, 8, (2, 64)), ("stream", 40, 4, 6, (1, 64))],
    "sincos": [("local", 4, 4, 0, (8, 32)), ("local", 2, 4, 0, (18, 14)), ("stream", 89, 4, 0, (4, 64)),
               ("stream", 134, 4, 0, (32, 8)), ("stream", 134, 4, 0, (1, 64)),
               ("stream", 134, 4, 0, (32, 8), -1, 1), ("stream", 89, 4, 0, (4, 64), -1, 1),
               ("stream", 67, 4, 0, (32, 8), -1, 1)],
}


def best_known_configuration(ls, torch, o, reps):
    """The fastest of the kernel's strong configurations on workload `o`, per application."""
    st = ls.Stencil.from_workload(o)
    a = torch.from_numpy(o.grid()).cuda()
    b = torch.empty_like(a)
    burst = sweep_burst(o)
    configs = STRONG_CONFIGS[o.kernel]
    mean, status, best = st.sweep_configs(a, b, configs, iters=burst, reps=reps)
    st.close()
    del a, b
    if best < 0:
        return None
    c = configs[best]
    per_app_ms = mean[best] / burst
    fused = max(1, c[3])
    # a launch moves the matrix once whatever it fuses: bytes per launch over the launch's time
    gbs = o.cells * o.bytes_per_cell_update / (per_app_ms * fused) / 1e6
    return {"mapping": mapping_name((c[0], c[1], c[2]) + ((c[3],) if c[3] else ())), "wg": list(c[4]),
            "nt_store": c[6] if len(c) > 6 else 0, "applications_per_launch": fused, "ms_per_application": per_app_ms,
            "gcells_s": o.cells / per_app_ms / 1e6, "algorithmic_gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
            "configurations_swept": len(configs)}


# one application of the heat step on matrices that no cache holds (256 MiB and 1 GiB each way): the
# workgroup sizes that win there are not those of the 4096^2 matrix, and the workgroup numbering and
# non-temporal output stores matter the other way round - the reason to sweep per dataset
LARGE_HEAT_CONFIGS = [(m, cr, 4, 0, wg, remap, nt)
                      for m, cr in (("direct", 2), ("direct", 4), ("local", 2), ("local", 4))
                      for wg in ((4, 16), (4, 64), (2, 256), (8, 64), (1, 512))
                      for remap in (1, 0) for nt in (0, 1)]


def larger_matrices(ls, wl, torch, reps):
    out = {}
    for n in (8192, 16384):
        o = wl.config(3, rows=n, cols=n, iters=1)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(o.seed)
        a = torch.rand(n * n, generator=gen, device="cuda", dtype=torch.float32) * 100.0
        b = torch.empty_like(a)
        st = ls.Stencil.from_workload(o)
        burst = 4
        mean, status, best = st.sweep_configs(a, b, LARGE_HEAT_CONFIGS, iters=burst, reps=reps)
        copy_ms, _ = ls.time_copy(a, b, burst=burst, reps=reps)
        fixed = LARGE_HEAT_CONFIGS.index(("direct", 2, 4, 0, (4, 16), 1, 0))   # the 4096^2 matrix's best
        st.close()
        del a, b
        c = LARGE_HEAT_CONFIGS[best]
        gbs = lambda ms: n * n * 8 / (ms / burst) / 1e6
        out["heat %dx%d" % (n, n)] = {
            "best": {"mapping": mapping_name(c[:3]), "wg": list(c[4]), "xcd_remap": c[5], "nt_store": c[6]},
            "ms_per_application": mean[best] / burst, "algorithmic_gbs": gbs(mean[best]),
            "frac_of_hbm_peak": gbs(mean[best]) / HBM_PEAK_GBS,
            "with_the_4096_best": {"algorithmic_gbs": gbs(mean[fixed]), "frac_of_hbm_peak": gbs(mean[fixed]) / HBM_PEAK_GBS},
            "copy_kernel_gbs": 2.0 * n * n * 4 / copy_ms / 1e6, "configurations_swept": len(LARGE_HEAT_CONFIGS)}
    return out


def leave_one_out_prediction(ls, wl, torch, index, mapping_of, reps):
    """Section 7's leave-one-out evaluation in miniature: sweep the other four workloads, train
    the classifier on their (f(s), Omega(s)) pairs, predict for workload `index` with the
    NearestNeighbour fallback of Algorithm 1.  Returns (predicted size, training table)."""
    pred = ls.Predictor()
    table = []
    for i in range(5):
        if i == index:
            continue
        o = wl.config(i)
        st = ls.Stencil.from_workload(o)
        st.set_mapping(*mapping_of(o))
        st.set_option(ls.OPT_SWEEP_CUTOFF, 300)      # training sweeps: adaptive sampling
        a = torch.from_numpy(o.grid()).cuda()
        b = torch.empty_like(a)
        burst = sweep_burst(o)
        res = st.sweep(a, b, o.wg_sizes(), iters=burst, fixed=(0, 0), reps=reps)
        if res.best:
            pred.add(st.features(), res.best)
            per_app_ms = res.best_ms / burst
            table.append({"workload": o.name.split()[0], "oracle_wg": list(res.best),
                          "mapping": mapping_name(mapping_of(o)), "ms_per_application": per_app_ms,
                          "gcells_s": o.cells / per_app_ms / 1e6,
                          "algorithmic_gbs": o.cells * o.bytes_per_cell_update / per_app_ms / 1e6,
                          "frac_of_hbm_peak": o.cells * o.bytes_per_cell_update / per_app_ms / 1e6 / HBM_PEAK_GBS})
        st.close()
        del a, b
    return pred, table


def recorded_traffic(kernel_label):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None when there is
    none for this kernel or the kernel sources have changed since the counters were taken."""
    from paper_1511_02490_amd import rocprof_summary as rs
    import re
    try:
        with open(rs.TRAFFIC_JSON) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    rec = table.get(kernel_label)
    if rec is None and kernel_label.startswith(("stream_kernel", "march_kernel")):
        # in the streaming kernels a wavefront's accesses do not depend on how wavefronts are grouped
        # into workgroups: a record taken with another workgroup size of the same mapping serves
        strip = lambda k: re.sub(r", wg \d+x\d+", "", k)
        rec = next((v for k, v in sorted(table.items()) if strip(k) == strip(kernel_label)), None)
    if not rec or rec.get("source_hash") != rs.kernel_source_hash():
        return None
    return rec["traffic_bytes_per_launch"]


def cpu_baseline(wl_mod, w, target_seconds):
    """The oracle, as it stands, on the first rows of the workload's matrix for a bounded
    number of iterations (the sample is sized from a short calibration run)."""
    from oracle import stencil as oracle
    threads = oracle.max_threads()
    g = w.grid()
    rows = w.rows
    run = lambda it: oracle.apply(g, w.kernel, w.halo, w.border, w.pad, w.weights, w.scalars, it)
    oracle.apply(g[:64], w.kernel, w.halo, w.border, w.pad, w.weights, w.scalars, 1)   # load library, spawn threads
    iters, dt = 1, 0.0
    while True:
        t0 = time.perf_counter()
        run(iters)
        dt = time.perf_counter() - t0
        if dt >= target_seconds / 3 or iters >= w.iters:
            break
        iters = int(min(w.iters, max(2 * iters, iters * 0.8 * target_seconds / max(dt, 1e-3))))
    # the same oracle on one thread, on a sample a tenth the size (context for the threaded figure)
    it1 = max(1, iters // 10)
    rows1 = rows if iters >= 10 else max(64, rows // 10)
    g1 = g[:rows1]
    t0 = time.perf_counter()
    oracle.apply(g1, w.kernel, w.halo, w.border, w.pad, w.weights, w.scalars, it1, threads=1)
    dt1 = time.perf_counter() - t0
    oracle.apply(g[:8], w.kernel, w.halo, w.border, w.pad, w.weights, w.scalars, 1, threads=threads)   # thread count back
    return {
        "value": rows * w.cols * iters / dt / 1e9,
        "unit": "Gcells/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "whole %d x %d matrix, %d of %d iterations, %.1f s" % (w.rows, w.cols, iters, w.iters, dt),
        "single_thread": {"value": rows1 * w.cols * it1 / dt1 / 1e9, "unit": "Gcells/s", "cores": 1,
                          "sample": "first %d rows, %d iterations, %.1f s" % (rows1, it1, dt1)},
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1511_02490_amd import libstencil as ls
    from paper_1511_02490_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    index = int(args.workload[1]) - 1
    w = wl.config(index)
    sizes = w.wg_sizes()
    if args.quick:
        sizes = sizes[::5]
    g = w.grid()
    tin = torch.from_numpy(g).cuda()
    tout = torch.empty_like(tin)
    cells = w.rows * w.cols

    burst = sweep_burst(w)
    cells_per_sample = cells * burst

    steps = args.steps if args.steps > 0 else {0: 200, 1: 200, 2: 20, 3: 5, 4: 100}[index]
    warmup = args.warmup if args.warmup >= 0 else max(1, steps // 10)

    def copy_reference(n=20):
        """GB/s of the plain copy kernel on this matrix (read + write), timed like a sweep sample."""
        mean_ms, _ = ls.time_copy(tin, tout, burst=max(burst, 2), reps=n)
        return 2.0 * tin.numel() * tin.element_size() / (mean_ms * 1e-3) / 1e9

    if args.copy_only:
        gbs = copy_reference(max(steps, 20))
        print(json.dumps({"metric": "plain copy kernel GB/s (read+write)", "value": gbs, "unit": "GB/s",
                          "config": {"workload": w.name, "bytes_each_way": tin.numel() * tin.element_size()}}))
        return

    st = ls.Stencil.from_workload(w)
    sweeps, sweep_seconds, predictor, others = {}, 0.0, {}, {}
    if args.wg:
        wg = tuple(int(x) for x in args.wg.split(","))
        m = args.mapping.split(",") if args.mapping else ["local", "1", "1"]
        blocking = (m[0],) + tuple(int(x) for x in m[1:])
        apply_mapping(st, blocking)
        best = (float("nan"), blocking, wg)
        best1 = best
    else:
        t_sweep0 = time.perf_counter()
        best = None    # (ms per sample, mapping, wg) over every mapping
        best1 = None   # the same over the mappings that make one application per launch
        for mapping in MAPPINGS[w.kernel]:
            try:
                apply_mapping(st, mapping)
            except ls.StencilError:
                continue                 # a mapping this scenario does not have (border mode, region)
            res = st.sweep(tin, tout, sizes, iters=burst, fixed=(4, 4), reps=args.reps)
            summ, _ = sweep_summary(res, cells_per_sample)
            summ["w_max"] = st.max_wg_size()
            sweeps[mapping_name(mapping)] = summ
            if res.best and (best is None or res.best_ms < best[0]):
                best = (res.best_ms, mapping, res.best)
            if res.best and len(mapping) == 3 and (best1 is None or res.best_ms < best1[0]):
                best1 = (res.best_ms, mapping, res.best)
        sweep_seconds = time.perf_counter() - t_sweep0
        assert best is not None, "no legal workgroup size"
        _, blocking, wg = best
        apply_mapping(st, blocking)

        # Algorithm 1 on this scenario, for the best mapping's family and for the paper's
        # mapping: train on the other four workloads' sweeps, predict, repair an illegal
        # prediction (NearestNeighbour), and score it on this workload's own sweep table.
        if not args.no_predictor:
            for tag, mapping_of in (("fast", lambda o: FAST_MAPPING[o.kernel]), ("paper", lambda o: ("local", 1, 1))):
                pred, table = leave_one_out_prediction(ls, wl, torch, index, mapping_of, max(5, args.reps // 3))
                mine = mapping_of(w)
                apply_mapping(st, mine)
                res = st.sweep(tin, tout, sizes, iters=burst, fixed=(4, 4), reps=args.reps)
                p = st.predict(pred, sizes)
                t_p = res.ms_of(p)
                if math.isnan(t_p) and st.is_legal(*p):
                    t_p = st.sweep(tin, tout, [p], iters=burst, fixed=(0, 0), reps=args.reps).mean_ms[0]
                t4 = res.ms_of((4, 4))
                if tag == "fast":
                    others = {t["workload"]: {k: v for k, v in t.items() if k != "workload"} for t in table}
                pretrained = None
                if mine == ("local", 1, 1):
                    # the classifier shipped with the library (trained offline on the 128-scenario study,
                    # which contains this kernel on other matrix sizes and, for C4, on this one)
                    shipped = ls.pretrained_predictor("local,1,1")
                    q = st.predict(shipped, sizes)
                    shipped.close()
                    t_q = res.ms_of(q)
                    pretrained = {"predicted_wg": list(q),
                                  "performance": (res.best_ms / t_q) if not math.isnan(t_q) else None}
                predictor[tag] = {"mapping": mapping_name(mine), "pretrained": pretrained,
                                  "trained_on": [{"workload": t["workload"], "oracle_wg": t["oracle_wg"]} for t in table],
                                  "predicted_wg": list(p),
                                  "oracle_wg": list(res.best), "performance": res.best_ms / t_p,
                                  "speedup_over_4x4": (t4 / t_p) if not math.isnan(t4) else None}
            apply_mapping(st, blocking)
            # the other workloads with the fastest kernels known for them (any mapping)
            for i in range(5):
                if i != index:
                    o = wl.config(i)
                    others.setdefault(o.name.split()[0], {})["best_known"] = best_known_configuration(
                        ls, torch, o, max(5, args.reps // 3))

    def choose_stores(mapping, size):
        """Plain or non-temporal output stores for this configuration, whichever the sweep's clock
        prefers (forced by --nt-store); leaves the handle on that choice."""
        if args.nt_store is not None:
            nt = int(args.nt_store)
        elif args.wg or mapping[2] == 1:      # one cell per work-item: no 16-byte stores to switch
            nt = 0
        else:
            depth = mapping[3] if len(mapping) > 3 else 0
            pair = [(mapping[0], mapping[1], mapping[2], depth, size, -1, flag) for flag in (0, 1)]
            mean, status, pick = st.sweep_configs(tin, tout, pair, iters=burst, reps=args.reps)
            # plain stores unless the others win by more than the run-to-run noise
            nt = 1 if (status[0] == ls.OK and status[1] == ls.OK and mean[1] < 0.98 * mean[0]) else 0
        apply_mapping(st, mapping)
        st.set_option(ls.OPT_NT_STORE, nt)
        return nt

    def choose_stores_for_steps():
        """The same choice for the timed steps, made on whole steps (all iterations of the workload):
        a short burst does not show what the stores do to a long chain of dependent launches."""
        if args.nt_store is not None or args.wg or blocking[2] == 1:
            return choose_stores(blocking, wg)
        apply_mapping(st, blocking)
        took = []
        per_trial = 1
        for flag in (0, 1):
            st.set_option(ls.OPT_NT_STORE, flag)
            t_a = time.perf_counter()
            st.run(tin, tout, w.iters, wg)
            torch.cuda.synchronize()
            if flag == 0:     # a trial lasts a few milliseconds, so that the host's part does not decide
                per_trial = max(1, min(500, int(0.004 / max(time.perf_counter() - t_a, 1e-6))))
            trials = []
            for _ in range(3):
                t_a = time.perf_counter()
                for _ in range(per_trial):
                    st.run(tin, tout, w.iters, wg)
                torch.cuda.synchronize()
                trials.append(time.perf_counter() - t_a)
            took.append(min(trials))
        nt = 1 if took[1] < 0.98 * took[0] else 0
        st.set_option(ls.OPT_NT_STORE, nt)
        return nt

    nt_store = choose_stores_for_steps()
    for _ in range(warmup):
        st.run(tin, tout, w.iters, wg)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.run(tin, tout, w.iters, wg)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    value = cells * w.iters * steps / dt / 1e9

    # kernel launch duration by HIP events on the launch stream (the sweep's own clock).  A
    # launch moves the matrix once (read + write) whatever the number of applications it fuses.
    alg_bytes = cells * w.bytes_per_cell_update

    def kernel_roofline(mapping, size):
        nt = choose_stores(mapping, size)
        depth = mapping[3] if len(mapping) > 3 else 1
        k_res = st.sweep(tin, tout, [size], iters=burst, fixed=(0, 0), reps=max(args.reps, 30))
        launches = -(-burst // depth)
        kernel_ms = k_res.mean_ms[0] / launches
        achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
        family = {"local": "tile", "direct": "direct", "temporal": "temporal", "stream": "stream"}[mapping[0]]
        if mapping[0] == "stream" and len(mapping) == 3:
            family = "march"            # register streaming, one application per launch
        label = "%s_kernel<%s> %dx%d cells/work-item, wg %dx%d" % (
            family, w.kernel, mapping[1], mapping[2], size[0], size[1]) + (
            ", %d applications/launch" % depth if depth > 1 else "") + (", non-temporal stores" if nt else "")
        out = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
               "frac": achieved / HBM_PEAK_GBS, "traffic": recorded_traffic(label),
               "kernel": label, "kernel_ms": kernel_ms, "algorithmic_bytes_per_launch": alg_bytes,
               "applications_per_launch": depth, "nt_store": nt,
               "gcells_s": cells * depth / (kernel_ms * 1e-3) / 1e9}
        # kernels that vector arithmetic bounds rather than memory (the sin/cos stencil; fused
        # applications): algorithmic fp32 operations against the published vector peak
        flops = flops_per_cell_update(w)
        if flops and (w.kernel == "sincos" or depth > 1):
            tflops = flops * cells * depth / (kernel_ms * 1e-3) / 1e12
            alu = {"bound": "alu", "achieved": tflops, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                   "frac": tflops / FP32_VECTOR_PEAK_TFLOPS, "flops_per_cell_update": flops}
            if w.kernel == "sincos":
                # measured to be bound by vector-ALU issue in every mapping: the arithmetic view leads,
                # the memory view stays beside it
                hbm = {k: out[k] for k in ("bound", "achieved", "peak", "unit", "frac")}
                out.update(alu)
                out["hbm"] = hbm
            else:
                out["alu"] = alu
        return out

    # `roofline` prices the best kernel that makes ONE application per launch: that is the
    # kernel whose bytes are all compulsory.  A temporally blocked kernel moves the matrix once
    # per `depth` applications, so its per-launch figure says little about HBM; it is reported
    # beside it as `roofline_timed_kernel` when it is the one the timed steps used.
    roofline_timed = None
    if len(blocking) > 3 and best1 is not None:
        roofline = kernel_roofline(best1[1], best1[2])
        roofline_timed = kernel_roofline(blocking, wg)
        roofline["note"] = ("single-application kernel; the timed steps used the temporally blocked kernel "
                            "in roofline_timed_kernel")
    else:
        roofline = kernel_roofline(blocking, wg)
    roofline["copy_kernel_gbs"] = copy_reference()
    apply_mapping(st, blocking)
    st.set_option(ls.OPT_NT_STORE, nt_store)

    larger = larger_matrices(ls, wl, torch, max(5, args.reps // 3)) if (index == 3 and not args.wg and not args.quick) else {}

    out = {
        "metric": "Gcells/s at best swept workgroup size (achieved HBM GB/s in roofline)",
        "value": value, "unit": "Gcells/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "rows": w.rows, "cols": w.cols, "iters": w.iters,
                   "halo_nsew": list(w.halo), "border": w.border, "best_wg": list(wg),
                   "staging": blocking[0], "cells_per_work_item": list(blocking[1:3]),
                   "applications_per_launch": blocking[3] if len(blocking) > 3 else 1,
                   "nt_store": nt_store, "sweep_burst": burst, "sweep_reps": args.reps},
        "roofline": roofline,
        "roofline_timed_kernel": roofline_timed,
        "sweep": {"seconds": sweep_seconds, "by_blocking": sweeps},
        "predictor": predictor,
        "other_workloads": others,
        "larger_matrices": larger,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, w, args.cpu_seconds)
    st.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
