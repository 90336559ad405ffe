"""The paper's experiment in miniature, on one MI355X: sweep the workgroup-size space of a set
of synthetic and real stencil scenarios (Section 5), then evaluate workgroup-size prediction
(Algorithm 1: nearest-neighbour and decision-tree classifiers over f(s) with the NearestNeighbour
fallback; Algorithm 2: nearest-neighbour and random-forest regressors on runtimes and on speedups) against
the sweep's oracle sizes with the metrics of Section 7.

    python -m paper_1511_02490_amd.autotune_study [--synthetic 32] [--reps 5] [--mapping local,1,1 | best]

`--mapping best` extends the space by the kernel family: every scenario is first timed under each
mapping the library has for it (local-memory tiles of 1x1, 2x4 and 4x4 cells per work-item, the direct
kernel, the register-marching kernel at a few segment heights) on a short list of workgroup sizes, and
the full sweep of workgroup sizes then runs under the fastest one, which the report names.

A large study can be split: `--json FILE --sweep-only` on the GPU records the sweeps, `--from-json
FILE` (same --synthetic and --mapping) evaluates them anywhere - legality, features and the
predictors make no GPU call.  `--export-training FILE` writes the (f(s), oracle size) pairs of the
sweeps as text: the files under tuning_data/ that `stencil_predictor_load` reads were made so.

Everything measured goes through the C ABI (sweeps, legality, features, predictor, baseline);
this script only builds the scenario list and the tables.  Prints a markdown report.
"""
from __future__ import annotations

import argparse
import json
import math
import statistics
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--synthetic", type=int, default=32)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--mapping", default="local,1,1")
    ap.add_argument("--fresh-matrices", action="store_true",
                    help="sweep single-application scenarios over a rotation of matrix pairs (about 512 MiB between two "
                         "uses of a pair), so that no sample finds its input in the last-level cache")
    ap.add_argument("--json", default="", help="also write the raw sweep tables here")
    ap.add_argument("--sweep-only", action="store_true", help="stop after the sweeps (with --json)")
    ap.add_argument("--from-json", default="", help="evaluate sweeps recorded with --json instead of sweeping")
    ap.add_argument("--export-training", default="",
                    help="write the (f(s), oracle size) pairs here (the data libstencil.pretrained_predictor loads) and stop")
    a = ap.parse_args()

    from paper_1511_02490_amd import libstencil as ls
    from paper_1511_02490_amd import workloads as wl

    pick_best = a.mapping == "best"
    m = "local,1,1".split(",") if pick_best else a.mapping.split(",")
    mapping = (m[0], int(m[1]), int(m[2]))
    # the mappings tried per scenario under `best`, and the sizes each is tried on
    candidates = [("local", 1, 1), ("local", 2, 4), ("local", 4, 4), ("direct", 2, 4), ("direct", 4, 4),
                  ("stream", 16, 4), ("stream", 32, 4), ("stream", 64, 4), ("stream", 128, 4)]
    probe_sizes = [(4, 64), (8, 32), (16, 16), (2, 32), (1, 64), (2, 128)]

    def use(st, mp):
        """Puts a scenario on a mapping, or on the paper's own where the library has no such kernel for it."""
        try:
            st.set_mapping(*mp)
            return tuple(mp)
        except ls.StencilError:
            st.set_mapping("local", 1, 1)
            return ("local", 1, 1)
    sizes = ls.enumerate_wg("pow2", 1024)
    scen = wl.synthetic_scenarios(a.synthetic) + wl.real_scenarios()
    kind = ["synthetic"] * a.synthetic + ["real"] * (len(scen) - a.synthetic)

    feats, times, status, mappings = [], [], [], []
    t0 = time.perf_counter()
    recorded = None
    if a.from_json:
        with open(a.from_json) as fh:
            recorded = json.load(fh)
        if recorded["scenarios"] != [w.name for w in scen] or [tuple(x) for x in recorded["sizes"]] != sizes \
                or recorded.get("mapping", a.mapping) != a.mapping:
            raise SystemExit("%s was recorded for another scenario list, size list or mapping" % a.from_json)
        times, status = recorded["times_ms"], recorded["status"]
        mappings = [tuple(mp) for mp in recorded.get("mappings", [])]
        a.reps = recorded.get("reps", a.reps)
        for w in scen:            # f(s) needs no GPU: taken afresh, so that recorded sweeps outlive a change of features
            st = ls.Stencil.from_workload(w)
            feats.append(st.features())
            st.close()
    else:
        import torch
    for w in ([] if recorded else scen):
        st = ls.Stencil.from_workload(w)
        tin = torch.from_numpy(w.grid()).cuda()
        tout = torch.empty(tin.shape, dtype=torch.uint8 if w.out_dtype == "u8" else tin.dtype, device="cuda")
        if a.fresh_matrices and w.iters == 1:
            pair_bytes = tin.numel() * tin.element_size() + tout.numel() * tout.element_size()
            n_pairs = int(min(24, max(3, 1 + math.ceil((512 << 20) / pair_bytes))))
            st.set_sweep_rotation([(tin, tout)] + [(tin.clone(), torch.empty_like(tout)) for _ in range(n_pairs - 1)])
        chosen = mapping
        if pick_best:
            best_ms = float("inf")
            for mp in candidates:
                if mp[1] > w.rows or use(st, mp) != mp:
                    continue
                probe = st.sweep(tin, tout, probe_sizes, iters=max(1, min(w.iters, 10)), fixed=(0, 0), reps=3)
                if probe.best is not None and probe.best_ms < best_ms:
                    best_ms, chosen = probe.best_ms, mp
        mappings.append(use(st, chosen))
        res = st.sweep(tin, tout, sizes, iters=max(1, min(w.iters, 10)), fixed=(0, 0), reps=a.reps)
        feats.append(st.features())
        times.append(res.mean_ms)
        status.append(res.status)
        st.close()
        del tin, tout
        print("swept %-44s %-14s best %-10s %.4f ms  refused %d" % (w.name, "%s %dx%d" % mappings[-1], res.best, res.best_ms,
                                                                   sum(1 for s in res.status if s != 0)),
              file=sys.stderr, flush=True)
    sweep_s = recorded["sweep_seconds"] if recorded else time.perf_counter() - t0
    if a.json and not recorded:
        with open(a.json, "w") as fh:
            json.dump({"sizes": sizes, "scenarios": [w.name for w in scen], "times_ms": times, "status": status,
                       "features": feats, "mapping": a.mapping, "mappings": mappings, "reps": a.reps,
                       "sweep_seconds": sweep_s}, fh)
    if a.sweep_only:
        return

    n_s, n_w = len(scen), len(sizes)
    nan = float("nan")
    if len(mappings) != n_s:               # sweeps recorded before the mapping was kept per scenario
        mappings = [mapping] * n_s
    oracle, perf = [], []
    for i in range(n_s):
        b, p, _ = ls.sweep_reduce(sizes, times[i], status[i], nan)
        oracle.append(b)
        perf.append(p)
    if a.export_training:
        # stencil_predictor_load's format: "features <n>", then n feature values and the oracle size per line
        with open(a.export_training, "w") as fh:
            fh.write("# (f(s), oracle workgroup size) pairs: device MI355X, mapping %s, %d samples per size, %d scenarios\n"
                     % (a.mapping, a.reps, sum(1 for i in range(n_s) if oracle[i] >= 0)))
            fh.write("# scenario i of the study's list is named in the comment above its line\n")
            fh.write("features %d\n" % len(feats[0]))
            for i in range(n_s):
                if oracle[i] >= 0:
                    fh.write("# %s\n" % scen[i].name)
                    fh.write(" ".join("%.17g" % x for x in feats[i]) + " %d %d\n" % tuple(sizes[oracle[i]]))
        return
    base = ls.baseline_wg(perf)                      # best fixed size that is legal everywhere
    idx = {s: j for j, s in enumerate(sizes)}

    def progress(what, done, of):
        if done == of or done % 10 == 0:
            print("evaluated %s: %d of %d" % (what, done, of), file=sys.stderr, flush=True)

    def evaluate(train, test, predictor_kind):
        rows = []
        for n_done, i in enumerate(test):
            progress(predictor_kind, n_done, len(test))
            tr = [k for k in train if k != i]
            if predictor_kind == "zeror":
                j = base
                legal_first = True
            else:
                pred = ls.Predictor(predictor_kind)
                for k in tr:
                    pred.add(feats[k], sizes[oracle[k]])
                raw = pred.classify(feats[i])
                st = ls.Stencil.from_workload(scen[i])
                use(st, mappings[i])
                legal_first = st.is_legal(*raw)
                j = idx[st.predict(pred, sizes)]
                st.close()
                pred.close()
            t = times[i][j]
            rows.append({"scenario": scen[i].name, "oracle": sizes[oracle[i]], "predicted": sizes[j],
                         "accurate": j == oracle[i], "valid_first": legal_first, "performance": perf[i][j],
                         "speedup_over_baseline": times[i][base] / t,
                         "speedup_over_4x4": times[i][idx[(4, 4)]] / t if status[i][idx[(4, 4)]] == 0 else nan,
                         "speedup_over_32x4": times[i][idx[(32, 4)]] / t if status[i][idx[(32, 4)]] == 0 else nan})
        return rows

    def evaluate_regression(train, test, target, model="nearest"):
        """Algorithm 2 with a regressor trained on runtimes (target = "runtime", fitness 1/x) or on
        speedups over the baseline size (target = "speedup", fitness x); model = "nearest"
        (nearest-neighbour regression) or "forest" (Section 5's random forest of regression trees:
        30 trees, seeded bootstrap samples and input subsets, leaves of two tuples or more)."""
        rows = []
        for n_done, i in enumerate(test):
            progress("%s regressor on %s" % (model, target), n_done, len(test))
            reg = ls.Regressor()
            n_tuples = 0
            for k in train:
                if k == i:
                    continue
                for j, w in enumerate(sizes):
                    if status[k][j] == 0:
                        y = times[k][j] if target == "runtime" else times[k][base] / times[k][j]
                        reg.add(feats[k], w, y)
                        n_tuples += 1
            if model == "forest":
                bootstrap, masks = wl.forest_draws(30, n_tuples, len(feats[i]) + 2, seed=wl.BASE_SEED + 200 + i)
                reg.fit_forest(bootstrap, masks, min_leaf=2, max_depth=32)
            st = ls.Stencil.from_workload(scen[i])
            use(st, mappings[i])
            (wr, wc), struck = st.predict_regression(reg, sizes, "reciprocal" if target == "runtime" else "identity")
            st.close()
            reg.close()
            j = idx[(wr, wc)]
            t = times[i][j]
            rows.append({"scenario": scen[i].name, "oracle": sizes[oracle[i]], "predicted": sizes[j],
                         "accurate": j == oracle[i], "valid_first": struck == 0, "performance": perf[i][j],
                         "speedup_over_baseline": times[i][base] / t,
                         "speedup_over_4x4": times[i][idx[(4, 4)]] / t if status[i][idx[(4, 4)]] == 0 else nan,
                         "speedup_over_32x4": times[i][idx[(32, 4)]] / t if status[i][idx[(32, 4)]] == 0 else nan})
        return rows

    def summary(rows):
        f = lambda key: [r[key] for r in rows if not math.isnan(r[key])]
        return {"n": len(rows), "accuracy": sum(r["accurate"] for r in rows) / len(rows),
                "valid_first": sum(r["valid_first"] for r in rows) / len(rows),
                "mean_performance": statistics.mean(f("performance")),
                "median_speedup_over_baseline": statistics.median(f("speedup_over_baseline")),
                "mean_speedup_over_baseline": statistics.mean(f("speedup_over_baseline")),
                "median_speedup_over_4x4": statistics.median(f("speedup_over_4x4")),
                "median_speedup_over_32x4": statistics.median(f("speedup_over_32x4"))}

    all_i = list(range(n_s))
    syn = [i for i in all_i if kind[i] == "synthetic"]
    real = [i for i in all_i if kind[i] == "real"]
    parts = {"leave-one-out, 1-NN + NearestNeighbour": evaluate(all_i, all_i, "nearest"),
             "leave-one-out, decision tree + NearestNeighbour": evaluate(all_i, all_i, "tree"),
             "leave-one-out, regressor on runtimes (Algorithm 2)": evaluate_regression(all_i, all_i, "runtime"),
             "leave-one-out, regressor on speedups (Algorithm 2)": evaluate_regression(all_i, all_i, "speedup"),
             "leave-one-out, random forest on runtimes (Algorithm 2)": evaluate_regression(all_i, all_i, "runtime", "forest"),
             "leave-one-out, random forest on speedups (Algorithm 2)": evaluate_regression(all_i, all_i, "speedup", "forest"),
             "ZeroR (always the baseline size)": evaluate(all_i, all_i, "zeror")}
    if syn and real:       # the paper's cross-validation: train on the synthetic scenarios, test on the real ones
        parts.update({
            "synthetic -> real, 1-NN + NearestNeighbour": evaluate(syn, real, "nearest"),
            "synthetic -> real, decision tree + NearestNeighbour": evaluate(syn, real, "tree"),
            "synthetic -> real, regressor on speedups (Algorithm 2)": evaluate_regression(syn, real, "speedup"),
            "synthetic -> real, random forest on speedups (Algorithm 2)": evaluate_regression(syn, real, "speedup", "forest")})

    worst_over_best = [max(t for t, s in zip(times[i], status[i]) if s == 0) / times[i][oracle[i]] for i in all_i]
    distinct = len({oracle[i] for i in all_i})
    refused = sum(1 for i in all_i for s in status[i] if s != 0)
    print("# Workgroup-size autotuning study on one MI355X")
    print()
    print("Mapping %s; %d scenarios (%d synthetic, %d real), %d workgroup sizes each (powers of two,"
          " product <= 1024), %d samples per size; sweep time %.0f s." % (
              "the fastest of the library's for each scenario (named in the table below)" if pick_best
              else "`%s %dx%d`" % mapping, n_s, len(syn), len(real), n_w, a.reps, sweep_s))
    if pick_best:
        count = {}
        for mp in mappings:
            count[mp[0]] = count.get(mp[0], 0) + 1
        print()
        print("* fastest mapping: " + ", ".join("%s for %d scenarios" % (k, v) for k, v in sorted(count.items())))
    print()
    if a.fresh_matrices:
        print("* single-application scenarios swept over a rotation of matrix pairs (fresh matrices)")
    print("* distinct oracle sizes: %d of %d scenarios; most common: %s" % (
        distinct, n_s, max(set(oracle), key=oracle.count) and sizes[max(set(oracle), key=oracle.count)]))
    print("* oracle over worst size: mean %.1fx (min %.2fx, max %.1fx)" % (
        statistics.mean(worst_over_best), min(worst_over_best), max(worst_over_best)))
    print("* refused test cases: %d of %d (%.1f %%)" % (refused, n_s * n_w, 100.0 * refused / (n_s * n_w)))
    print("* baseline (best size legal for every scenario, by geometric mean of performance): %s, reaching"
          " %.0f %% of the oracle's performance on average" % (
              sizes[base] if base >= 0 else None, 100 * statistics.mean(perf[i][base] for i in all_i)))
    print()
    print("| evaluation | n | accuracy | legal at first try | mean performance (of oracle) | median speedup over baseline | mean | median over 4x4 | median over 32x4 |")
    print("|---|---|---|---|---|---|---|---|---|")
    for name, rows in parts.items():
        s = summary(rows)
        print("| %s | %d | %.0f %% | %.0f %% | %.0f %% | %.2fx | %.2fx | %.2fx | %.2fx |" % (
            name, s["n"], 100 * s["accuracy"], 100 * s["valid_first"], 100 * s["mean_performance"],
            s["median_speedup_over_baseline"], s["mean_speedup_over_baseline"], s["median_speedup_over_4x4"],
            s["median_speedup_over_32x4"]))
    print()
    print("| scenario | mapping | oracle size | oracle ms | GB/s read + written | predicted (leave-one-out) | performance |")
    print("|---|---|---|---|---|---|---|")
    for i, r in enumerate(parts["leave-one-out, 1-NN + NearestNeighbour"]):
        w = scen[i]
        per_sweep_sample = max(1, min(w.iters, 10))
        gbs = w.cells * w.bytes_per_cell_update * per_sweep_sample / (times[i][oracle[i]] * 1e-3) / 1e9
        print("| %s | %s %dx%d | %dx%d | %.4f | %.0f | %dx%d | %.2f |" % (
            (r["scenario"],) + tuple(mappings[i]) + (r["oracle"][0], r["oracle"][1], times[i][oracle[i]], gbs,
                                                    r["predicted"][0], r["predicted"][1], r["performance"])))


if __name__ == "__main__":
    main()
