"""Condenses rocprofv3 output of a bench.py run into a short text summary and a traffic record.

    python -m paper_1511_02490_amd.rocprof_summary --prefix c4 --dir prof_out \
        --kernel direct_kernel --title "..." --command "..." > profiles/<name>.md

expects <dir>/<prefix>_trace (from --kernel-trace --stats), <dir>/<prefix>_fetch (--pmc FETCH_SIZE)
and <dir>/<prefix>_write (--pmc WRITE_SIZE), each produced with --output-format csv, plus the
bench.py JSON line in <dir>/<prefix>_trace.log.  HBM traffic is each counter's mean per dispatch
of the stencil kernel, scaled by (known bytes of the plain copy kernel / what the same counter
reads for it) from the same run.  With --record it also updates profiles/traffic.json, which
bench.py reports as `roofline.traffic` for as long as the kernel sources are unchanged.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")


def kernel_source_hash() -> str:
    """Hash of everything that shapes the device code and its launches (host_tuning.h is arithmetic
    on the host around the sweep: the predictors, the statistics)."""
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        if os.path.basename(f) == "host_tuning.h":
            continue
        with open(f, "rb") as fh:
            h.update(os.path.basename(f).encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def _one(pattern):
    hits = glob.glob(pattern)
    if len(hits) != 1:
        raise SystemExit("expected one file matching %s, found %d" % (pattern, len(hits)))
    return hits[0]


def counter_means(path, counter):
    """mean counter value per dispatch, keyed by kernel name"""
    acc = {}
    with open(path) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] != counter:
                continue
            acc.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def pick(d, needle):
    ks = [k for k in d if needle in k]
    if len(ks) != 1:
        raise SystemExit("kernel %r: %d matches in %s" % (needle, len(ks), list(d)))
    return ks[0]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dir", required=True)
    ap.add_argument("--prefix", required=True)
    ap.add_argument("--kernel", required=True, help="substring naming the stencil kernel")
    ap.add_argument("--title", default="")
    ap.add_argument("--command", default="", help="the bench.py arguments the three runs used")
    ap.add_argument("--record", action="store_true",
                    help="store the traffic in profiles/traffic.json under the kernel's label")
    a = ap.parse_args()
    d, p = a.dir, a.prefix

    stats = {}
    with open(_one(os.path.join(d, p + "_trace", "*kernel_stats.csv"))) as fh:
        for r in csv.DictReader(fh):
            stats[r["Name"]] = r
    bench = None
    with open(os.path.join(d, p + "_trace.log")) as fh:
        for line in fh:
            if line.startswith("{"):
                bench = json.loads(line)
    fetch = counter_means(_one(os.path.join(d, p + "_fetch", "*counter_collection.csv")), "FETCH_SIZE")
    write = counter_means(_one(os.path.join(d, p + "_write", "*counter_collection.csv")), "WRITE_SIZE")

    k = pick(stats, a.kernel)
    kc = pick(stats, "copy_kernel")
    roof = bench["roofline"]
    hbm = roof.get("hbm") or roof       # the memory view (kernels that arithmetic bounds carry it beside)
    copy_kib = bench["config"]["rows"] * bench["config"]["cols"] * (4 if bench["dtype"] == "f32" else 1) / 1024.0
    f_scale = copy_kib / fetch[pick(fetch, "copy_kernel")][0]
    w_scale = copy_kib / write[pick(write, "copy_kernel")][0]
    f_kib = fetch[pick(fetch, a.kernel)][0] * f_scale
    w_kib = write[pick(write, a.kernel)][0] * w_scale
    traffic = (f_kib + w_kib) * 1024.0

    out = []
    out.append("# %s" % (a.title or k))
    out.append("")
    out.append("Commands (from the repository root on the GPU box; `cd /tmp && export TMPDIR=/tmp` first):")
    out.append("")
    for flags, tag in (("--kernel-trace --stats", "trace"), ("--pmc FETCH_SIZE", "fetch"), ("--pmc WRITE_SIZE", "write")):
        out.append("    rocprofv3 %s --output-format csv -d %s/%s_%s -o %s -- python3 bench.py %s"
                   % (flags, d.rstrip("/"), p, tag, p, a.command))
    out.append("")
    out.append("## Kernel trace (--kernel-trace --stats)")
    out.append("")
    out.append("| kernel | calls | average ns | min ns | max ns | % of GPU time |")
    out.append("|---|---|---|---|---|---|")
    for name in (k, kc):
        r = stats[name]
        out.append("| `%s` | %s | %.0f | %s | %s | %s |" % (name.rsplit("(", 1)[0][:110], r["Calls"], float(r["AverageNs"]),
                                                          r["MinNs"], r["MaxNs"], r["Percentage"]))
    out.append("")
    out.append("bench.py's own clock in the same run (HIP events on the launch stream): kernel %.0f ns per launch, "
               "%.0f GB/s of algorithmic bytes (%d bytes per launch) = %.3f of the %.0f GB/s HBM peak; "
               "plain copy kernel on the same matrix: %.0f GB/s."
               % (roof["kernel_ms"] * 1e6, hbm["achieved"], roof["algorithmic_bytes_per_launch"], hbm["frac"],
                  hbm["peak"], roof["copy_kernel_gbs"]))
    if "hbm" in roof:
        out.append("")
        out.append("bench.py reports this kernel as bound by vector arithmetic: %.1f TFLOP/s of algorithmic fp32 "
                   "operations (%d per cell) = %.3f of the published %.1f TFLOP/s vector peak."
                   % (roof["achieved"], roof["flops_per_cell_update"], roof["frac"], roof["peak"]))
    if float(stats[k]["AverageNs"]) < 15000.0:
        out.append("")
        out.append("(A kernel this short finishes faster than the host can issue the next launch while the profiler "
                   "intercepts every call, so in a profiled run the event-timed figure includes idle gaps between "
                   "launches; the trace's average is the kernel's own duration and agrees with bench.py's clock in "
                   "an unprofiled run.)")
    out.append("")
    out.append("## HBM traffic counters (--pmc, one counter per run)")
    out.append("")
    out.append("| counter | stencil kernel, KiB / dispatch | copy kernel, KiB / dispatch | copy kernel moves | scale | stencil, scaled KiB |")
    out.append("|---|---|---|---|---|---|")
    out.append("| FETCH_SIZE | %.1f | %.1f | %.0f KiB | %.4f | %.1f |" % (
        fetch[pick(fetch, a.kernel)][0], fetch[pick(fetch, "copy_kernel")][0], copy_kib, f_scale, f_kib))
    out.append("| WRITE_SIZE | %.1f | %.1f | %.0f KiB | %.4f | %.1f |" % (
        write[pick(write, a.kernel)][0], write[pick(write, "copy_kernel")][0], copy_kib, w_scale, w_kib))
    out.append("")
    out.append("Traffic per launch: %.0f bytes (read %.1f KiB + write %.1f KiB) against %d algorithmic bytes: ratio %.4f."
               % (traffic, f_kib, w_kib, roof["algorithmic_bytes_per_launch"],
                  traffic / roof["algorithmic_bytes_per_launch"]))
    print("\n".join(out))

    if a.record:
        rec = {}
        if os.path.exists(TRAFFIC_JSON):
            with open(TRAFFIC_JSON) as fh:
                rec = json.load(fh)
        rec[roof["kernel"]] = {"workload": bench["config"]["workload"], "traffic_bytes_per_launch": traffic,
                         "fetch_kib": f_kib, "write_kib": w_kib, "fetch_scale": f_scale, "write_scale": w_scale,
                         "source_hash": kernel_source_hash()}
        with open(TRAFFIC_JSON, "w") as fh:
            json.dump(rec, fh, indent=1, sort_keys=True)
            fh.write("\n")
        print("recorded %r in %s" % (roof["kernel"], TRAFFIC_JSON), file=sys.stderr)


if __name__ == "__main__":
    main()
