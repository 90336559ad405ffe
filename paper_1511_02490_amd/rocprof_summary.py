"""Condenses rocprofv3 output of a bench.py run into a short text summary and a counter record.

    python -m paper_1511_02490_amd.rocprof_summary --prefix c5march --dir gpurun_out/prof \
        --kernel march_kernel --title "..." --command "<bench.py arguments>" --record > profiles/<name>.md

expects, each produced with --output-format csv by the commands the summary prints:
  <dir>/<prefix>_trace  (--kernel-trace --stats) and the bench.py JSON line in <dir>/<prefix>_trace.log,
  <dir>/<prefix>_fetch  (--pmc FETCH_SIZE), <dir>/<prefix>_write (--pmc WRITE_SIZE),
  and optionally <dir>/<prefix>_pmcA, <dir>/<prefix>_pmcB (--pmc with the counter lists below).
HBM traffic is each counter's mean per dispatch of the stencil kernel, scaled by (known bytes of
the plain copy kernel / what the same counter reads for it) from the same run.  With --record it
also updates profiles/traffic.json, which bench.py reports (`roofline.traffic`, `roofline.valu_issue`)
for as long as the sources of that kernel family are unchanged.
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

# the two counter passes beyond FETCH_SIZE / WRITE_SIZE (one --pmc run holds at most 8 SQ_ and 2 GRBM_ counters)
PMC_PASSES = {
    "pmcA": "SQ_INSTS_VALU SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES SQ_WAVES SQ_WAVE_CYCLES SQ_INSTS_VALU_TRANS_F32 "
            "SQ_INSTS_SALU GRBM_GUI_ACTIVE",
    "pmcB": "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_ACTIVE_INST_LDS SQ_WAIT_INST_LDS "
            "SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_WAIT_INST_ANY",
}
N_SIMD = 256 * 4            # SIMD units of an MI355X
N_SHADER_ENGINES = 32       # SQ_BUSY_CYCLES is summed over them

# source files that shape each kernel family's device code and launches
_COMMON = ["stencil_ops.h", "tile_kernel.h", "variants.h"]
FAMILY_SOURCES = {
    "tile": _COMMON,
    "direct": _COMMON + ["direct_kernel.h"],
    "temporal": _COMMON + ["temporal_kernel.h"],
    "stream": _COMMON + ["stream_kernel.h", "life_stream_kernel.h"],
    "march": _COMMON + ["march_kernel.h", "march_masked_kernel.h"],
}


def family_of(label: str) -> str:
    """Kernel family of a label like 'C5: march_kernel<sincos> 134x4 cells/work-item, wg 32x8'."""
    for fam in FAMILY_SOURCES:
        if fam + "_kernel<" in label:
            return fam
    raise ValueError("no kernel family in %r" % label)


def kernel_source_hash(family: str) -> str:
    """Hash of the sources of one kernel family and of the compiler flags."""
    h = hashlib.sha256()
    for name in sorted(set(FAMILY_SOURCES[family])):
        with open(os.path.join(HERE, "csrc", name), "rb") as fh:
            h.update(name.encode() + b"\0" + fh.read())
    from paper_1511_02490_amd import build
    h.update(" ".join(build.HIPCC_FLAGS).encode())
    return h.hexdigest()[:16]


def _one(pattern):
    hits = glob.glob(pattern)
    if len(hits) != 1:
        raise SystemExit("expected one file matching %s, found %d" % (pattern, len(hits)))
    return hits[0]


def counter_rows(path):
    """{kernel name: {counter: [values per dispatch]}} plus {kernel name: launch attributes}"""
    acc, attrs = {}, {}
    with open(path) as fh:
        for r in csv.DictReader(fh):
            acc.setdefault(r["Kernel_Name"], {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
            attrs[r["Kernel_Name"]] = {"workgroup": r["Workgroup_Size"], "lds_bytes": r["LDS_Block_Size"],
                                       "vgprs": r["VGPR_Count"], "agprs": r["Accum_VGPR_Count"], "sgprs": r["SGPR_Count"],
                                       "scratch": r["Scratch_Size"], "grid": r["Grid_Size"]}
    return acc, attrs


def counter_means(path, counter):
    acc, _ = counter_rows(path)
    return {k: (sum(v[counter]) / len(v[counter]), len(v[counter])) for k, v in acc.items() if counter in v}


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
    ap.add_argument("--command", default="", help="the bench.py arguments the runs used")
    ap.add_argument("--record", action="store_true",
                    help="store traffic and instruction counts in profiles/traffic.json under the kernel's label")
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
    passes = {}
    for tag in PMC_PASSES:
        hits = glob.glob(os.path.join(d, p + "_" + tag, "*counter_collection.csv"))
        if len(hits) == 1:
            passes[tag] = counter_rows(hits[0])

    k = pick(stats, a.kernel)
    kc = pick(stats, "copy_kernel")
    roof = bench["roofline"]
    cfg = bench["config"]
    cells = cfg["rows"] * cfg["cols"]
    depth = roof["applications_per_launch"]
    # the plain copy kernel copies the input matrix: one element of the workload's type per cell
    copy_kib = cells * {"f32": 4, "i32": 4, "f64": 8, "u8": 1}[bench["dtype"]] / 1024.0
    f_scale = copy_kib / fetch[pick(fetch, "copy_kernel")][0]
    w_scale = copy_kib / write[pick(write, "copy_kernel")][0]
    f_kib = fetch[pick(fetch, a.kernel)][0] * f_scale
    w_kib = write[pick(write, a.kernel)][0] * w_scale
    traffic = (f_kib + w_kib) * 1024.0
    avg_ns = float(stats[k]["AverageNs"])

    out = []
    out.append("# %s" % (a.title or k))
    out.append("")
    out.append("Commands (from the repository root on the GPU box, after `python -c \"import __graft_entry__ as g; "
               "g.build()\"`; `cd /tmp && export TMPDIR=/tmp` first, paths then relative to the repository):")
    out.append("")
    runs = [("--kernel-trace --stats", "trace"), ("--pmc FETCH_SIZE", "fetch"), ("--pmc WRITE_SIZE", "write")]
    runs += [("--pmc " + PMC_PASSES[tag], tag) for tag in passes]
    for flags, tag in runs:
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
    out.append("Algorithmic bytes per launch: %d (%d cells x %d B); over the trace's average duration: %.0f GB/s = %.3f "
               "of the 8000 GB/s HBM peak (over its minimum: %.3f)."
               % (roof["algorithmic_bytes_per_launch"], cells, roof["algorithmic_bytes_per_launch"] // cells,
                  roof["algorithmic_bytes_per_launch"] / avg_ns, roof["algorithmic_bytes_per_launch"] / avg_ns / 8000.0,
                  roof["algorithmic_bytes_per_launch"] / float(stats[k]["MinNs"]) / 8000.0))
    out.append("")
    out.append("bench.py's own clock in the same run (HIP events on the launch stream): kernel %.0f ns per launch, "
               "%.0f GB/s = %.3f of the peak; %d timed steps at %.4f ms per step (%d launches each); plain copy kernel "
               "on the same matrix: %.0f GB/s."
               % (roof["kernel_ms"] * 1e6, roof["achieved"], roof["frac"], bench["steps"], bench["ms_per_step"],
                  -(-cfg["iters"] // depth), roof["copy_kernel_gbs"]))
    if avg_ns < 15000.0:
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

    derived = {}
    if passes:
        c, attrs = {}, {}
        for tag, (acc, at) in passes.items():
            kk = pick(acc, a.kernel)
            attrs = at[kk]
            for name, vals in acc[kk].items():
                c[name] = sum(vals) / len(vals)
        out.append("")
        out.append("## Instruction, occupancy and local-memory counters (--pmc, means per dispatch of the stencil kernel)")
        out.append("")
        out.append("Launch as rocprofv3 lists it: workgroup of %s work-items, grid of %s work-items, VGPR_Count %s (+%s "
                   "accumulation), SGPR_Count %s, LDS_Block_Size %s (the kernels' dynamically sized tile is not in that "
                   "column), Scratch_Size %s."
                   % (attrs["workgroup"], attrs["grid"], attrs["vgprs"], attrs["agprs"], attrs["sgprs"], attrs["lds_bytes"],
                      attrs["scratch"]))
        out.append("")
        out.append("| counter | per dispatch |")
        out.append("|---|---|")
        for name in sorted(c):
            out.append("| %s | %.6g |" % (name, c[name]))
        out.append("")
        updates = cells * depth
        lines = []
        if "SQ_INSTS_VALU" in c:
            derived["valu_insts_per_launch"] = c["SQ_INSTS_VALU"]
            derived["valu_trans_insts_per_launch"] = c.get("SQ_INSTS_VALU_TRANS_F32", 0.0)
            per = c["SQ_INSTS_VALU"] * 64.0 / updates
            slots = (c["SQ_INSTS_VALU"] + 3.0 * c.get("SQ_INSTS_VALU_TRANS_F32", 0.0)) * 64.0 / updates
            lines.append("vector instructions per cell update: %.2f (SQ_INSTS_VALU x 64 lanes / %d cell updates); issue slots per "
                         "cell update, a transcendental instruction holding its slot four times as long: %.2f" % (per, updates, slots))
            rate = slots * updates / (avg_ns * 1e-9)
            lines.append("issue rate over the trace's average duration: %.1f T lane-instructions/s = %.3f of 256 CUs x 4 SIMDs x "
                         "16 lanes x 2.4 GHz = 39.3 T/s" % (rate / 1e12, rate / (N_SIMD * 16 * 2.4e9)))
        if "SQ_BUSY_CYCLES" in c and "SQ_ACTIVE_INST_VALU" in c:
            cyc = c["SQ_BUSY_CYCLES"] / N_SHADER_ENGINES
            busy = c["SQ_ACTIVE_INST_VALU"] * 4.0 / (N_SIMD * cyc)
            derived["valu_busy_frac"] = busy
            lines.append("kernel cycles (SQ_BUSY_CYCLES / %d shader engines): %.0f, i.e. %.2f GHz over the trace's average duration; "
                         "vector ALUs busy (SQ_ACTIVE_INST_VALU x 4 cycles / (%d SIMDs x kernel cycles)): %.1f %%"
                         % (N_SHADER_ENGINES, cyc, cyc / avg_ns, N_SIMD, 100.0 * busy))
            if "SQ_WAVE_CYCLES" in c:
                occ = c["SQ_WAVE_CYCLES"] * 4.0 / (N_SIMD * cyc)
                derived["mean_waves_per_simd"] = occ
                lines.append("occupancy: %.0f wavefronts per launch, on average %.2f resident per SIMD (SQ_WAVE_CYCLES x 4 / "
                             "(%d SIMDs x kernel cycles))" % (c.get("SQ_WAVES", float("nan")), occ, N_SIMD))
        if c.get("SQ_LDS_IDX_ACTIVE"):
            derived["lds_bank_conflict_frac"] = c["SQ_LDS_BANK_CONFLICT"] / c["SQ_LDS_IDX_ACTIVE"]
            lines.append("local memory: %.3g instructions per dispatch; bank-conflict cycles / active cycles "
                         "(SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE): %.3f"
                         % (c.get("SQ_INSTS_LDS", float("nan")), derived["lds_bank_conflict_frac"]))
        elif "SQ_INSTS_LDS" in c:
            lines.append("local memory: not used (SQ_INSTS_LDS = %.0f)" % c["SQ_INSTS_LDS"])
        out.extend("* " + l for l in lines)
    print("\n".join(out))

    if a.record:
        rec = {}
        if os.path.exists(TRAFFIC_JSON):
            with open(TRAFFIC_JSON) as fh:
                rec = json.load(fh)
        entry = {"workload": cfg["workload"], "traffic_bytes_per_launch": traffic,
                 "fetch_kib": f_kib, "write_kib": w_kib, "fetch_scale": f_scale, "write_scale": w_scale,
                 "trace_average_ns": avg_ns, "source_hash": kernel_source_hash(family_of(roof["kernel"]))}
        entry.update(derived)
        rec[roof["kernel"]] = entry
        with open(TRAFFIC_JSON, "w") as fh:
            json.dump(rec, fh, indent=1, sort_keys=True)
            fh.write("\n")
        print("recorded %r in %s" % (roof["kernel"], TRAFFIC_JSON), file=sys.stderr)


if __name__ == "__main__":
    main()
