"""Turns the raw rocprofv3 output of three profiled `bench.py --lean` runs of one workload into the short
summary kept under profiles/ and into that workload's record of profiles/traffic.json (which bench.py reads
for `roofline.traffic`).

    python -m paper_2604_16883_amd.profile_summary <dir> <workload>

<dir> holds, as written by the commands the summary itself lists:
    trace/t_kernel_trace.csv, trace/t_kernel_stats.csv    rocprofv3 --kernel-trace --stats
    fetch/f_counter_collection.csv, fetch.log             rocprofv3 --pmc FETCH_SIZE and the run's stdout
    write/w_counter_collection.csv, write.log             rocprofv3 --pmc WRITE_SIZE and the run's stdout
    trace.log                                             stdout of the traced run (bench.py's JSON line)
    util/, insts/, tcc/ + util.log, insts.log, tcc.log    optional: three more --pmc runs (UTIL_PASSES) and their stdout
The partial kernel's dispatches are attributed to the benchmark's modes by order: the JSON line carries how
many launches each mode makes.  Counter units are scaled by the plain copy kernel of known size that every
bench run dispatches once.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 1 << 30          # bench.py's calibration copy: 1 GiB read + 1 GiB written

KERNELS = (("sr_partial", "sr_partial"), ("sr_combine", "sr_combine"), ("sr_probe_kernel", "sr_probe"),
           ("sr_anchor", "sr_anchor"), ("sr_copy_probe", "sr_copy_probe"), ("sr_read_probe", "sr_read_probe"))


def short(name: str):
    for key, label in KERNELS:
        if key in name:
            return label
    return None


def find(base: str, pattern: str) -> str:
    hits = sorted(glob.glob(os.path.join(base, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit("no %s under %s" % (pattern, base))
    return hits[0]


def bench_line(path: str) -> dict:
    for line in open(path):
        line = line.strip()
        if line.startswith("{") and '"metric"' in line:
            return json.loads(line)
    raise SystemExit("no benchmark JSON line in %s" % path)


def split_by_plan(values, plan):
    """plan: [label, launches of the mode, (optional) how many of them come before the first timed one]."""
    out, i = {}, 0
    for entry in plan:
        label, n = entry[0], entry[1]
        out[label] = values[i:i + n]
        i += n
    if i != len(values):
        raise SystemExit("dispatch plan covers %d launches, the profile has %d" % (i, len(values)))
    return out


def counters(path: str):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        s = short(r["Kernel_Name"])
        if s:
            d[s].append(float(r["Counter_Value"]))
    return d


def leading(plan, warmup):
    """Per mode, the dispatches in front of the first timed one (device preconditioning + warm-up steps): left out of means."""
    return {e[0]: (e[2] if len(e) > 2 else warmup) for e in plan}


def counter_table(path: str):
    """{(kernel, counter): [value per dispatch, in dispatch order]} of a counter_collection.csv that holds several
    counters; rows of one dispatch and counter (one per hardware instance) are summed."""
    acc = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        s = short(r["Kernel_Name"])
        if s:
            key = (s, r["Counter_Name"], int(r["Dispatch_Id"]))
            acc[key] = acc.get(key, 0.0) + float(r["Counter_Value"])
    out = collections.defaultdict(list)
    for (s, name, did) in sorted(acc, key=lambda k: k[2]):
        out[(s, name)].append(acc[(s, name, did)])
    return out


UTIL_PASSES = (("util", "MfmaUtil VALUBusy LDSBankConflict OccupancyPercent"),
               ("insts", "SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_VMEM_RD SQ_INSTS_LDS SQ_WAVES SQ_INSTS_SALU"),
               ("tcc", "TCC_HIT TCC_MISS TCC_REQ"))


def utilisation_section(base, wl, cmd_short, det):
    """Optional: utilisation, instruction and L2 counters of the partial kernel from three further runs (directories
    util/, insts/, tcc/ under <dir>, each with its own trace-free --pmc pass and its own bench line in <pass>.log)."""
    have = [(d, names) for d, names in UTIL_PASSES if glob.glob(os.path.join(base, d, "**", "*counter_collection.csv"), recursive=True)]
    if not have:
        return []
    out = ["", "## utilisation, instruction and L2 counters of the partial kernel (further runs, counters only)", ""]
    for d, names in have:
        out.append("    rocprofv3 --pmc %s --output-format csv -d $D/%s -o p -- %s > $D/%s.log" % (names, d, cmd_short, d))
    rows, labels = [], None
    for d, names in have:
        line = bench_line(os.path.join(base, d + ".log"))
        plan = line["detail"][wl]["dispatch_plan"]
        lead = leading(plan, line["warmup"])
        labels = [e[0] for e in plan]
        tab = counter_table(find(os.path.join(base, d), "*counter_collection.csv"))
        for name in names.split():
            vals = tab.get(("sr_partial", name))
            if not vals:
                continue
            per = split_by_plan(vals, plan)
            rows.append((name, [sum(per[l][lead[l]:]) / max(len(per[l][lead[l]:]), 1) for l in labels]))
    blocks = {l: max(det[l]["algorithmic_bytes"] // 32768, 1) for l in labels}      # 64-token blocks streamed, about
    out += ["", "Means per dispatch of the partial kernel (warm-up dispatches left out); blocks of 64 tokens streamed: " +
            ", ".join("%s %d" % (l, blocks[l]) for l in labels) + ".", "",
            "| counter | " + " | ".join(labels) + " |", "|---|" + "---|" * len(labels)]
    for name, vals in rows:
        out.append("| %s | %s |" % (name, " | ".join("%.4g" % v for v in vals)))
    by = dict(rows)
    if "SQ_INSTS_MFMA" in by and "SQ_INSTS_VALU" in by and "SQ_INSTS_VMEM_RD" in by:
        i = len(labels) - 1          # the dense mode streams the most blocks
        out += ["", "Per 64-token block (%s): %.0f MFMA, %.0f VALU and %.1f vector-memory read instructions per wavefront-block." % (
            labels[i], by["SQ_INSTS_MFMA"][i] / blocks[labels[i]], by["SQ_INSTS_VALU"][i] / blocks[labels[i]],
            by["SQ_INSTS_VMEM_RD"][i] / blocks[labels[i]])]
    if "TCC_REQ" in by and "TCC_HIT" in by:
        out += ["L2: %s requests of 128 bytes per dispatch, %s of them hits: a pure stream, nothing is re-read." % (
            " / ".join("%.3g" % v for v in by["TCC_REQ"]), " / ".join("%.1f %%" % (100 * h / max(r, 1)) for h, r in zip(by["TCC_HIT"], by["TCC_REQ"])))]
    return out


def main(argv):
    if len(argv) != 3:
        raise SystemExit(__doc__)
    base, wl = argv[1], argv[2]
    from bench import kernel_source_sha          # the same hash bench.py checks the record against
    line = bench_line(os.path.join(base, "trace.log"))
    det = line["detail"][wl]
    plan = det["dispatch_plan"]
    steps, warmup = line["steps"], line["warmup"]
    cmd = "python3 $R/bench.py --workload %s --lean --steps %d --warmup %d" % (wl, steps, warmup)
    out = ["# rocprofv3 summary: sr_partial_balanced_kernel and sr_combine_kernel, workload %s (%s, bf16)" % (wl, det["description"]), "",
           "Commands (run from /tmp with TMPDIR=/tmp on the MI355X box, R = repository root, D = a scratch directory for the raw output):", "",
           "    rocprofv3 --kernel-trace --stats --output-format csv -d $D/trace -o t -- %s > $D/trace.log" % cmd,
           "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $D/fetch -o f -- %s > $D/fetch.log" % cmd,
           "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $D/write -o w -- %s > $D/write.log" % cmd,
           "    python3 -m paper_2604_16883_amd.profile_summary $D %s" % wl, "",
           "Each run launches the modes below in this order; per mode 0.1 s of untimed calls (the device is idle at process start and "
           "runs slower for its first milliseconds of work), then %d warm-up + 1 queued + %d timed launches, 50 to 200 for the step-time spread and 100 "
           "with per-kernel HIP events.  The routing probe is fused into the partial kernel, so no sr_probe_kernel is dispatched.  sr_read_probe / "
           "sr_copy_probe are the benchmark's calibration kernels (2 GiB streaming read; 1 GiB copy of known traffic)."
           % (warmup, steps), "",
           "## kernel-trace --stats (durations in us, all dispatches of a kernel name)", "",
           "| kernel | calls | avg | min | max |", "|---|---|---|---|---|"]
    for r in csv.DictReader(open(find(base, "t_kernel_stats.csv"))):
        s = short(r["Name"])
        if s:
            out.append("| %s | %s | %.1f | %.1f | %.1f |" % (s, r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                                                          float(r["MaxNs"]) / 1e3))
    rows = sorted((r for r in csv.DictReader(open(find(base, "t_kernel_trace.csv")))), key=lambda r: int(r["Start_Timestamp"]))
    dur_p = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in rows if short(r["Kernel_Name"]) == "sr_partial"]
    dur_c = [(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in rows if short(r["Kernel_Name"]) == "sr_combine"]
    # gap between the end of a partial kernel and the start of the merge kernel that follows it
    gaps = []
    for a, b in zip(rows, rows[1:]):
        if short(a["Kernel_Name"]) == "sr_partial" and short(b["Kernel_Name"]) == "sr_combine":
            gaps.append((int(b["Start_Timestamp"]) - int(a["End_Timestamp"])) / 1e3)
    by_p, by_c, by_g = split_by_plan(dur_p, plan), split_by_plan(dur_c, plan), split_by_plan(gaps, plan)
    f, w = counters(find(base, "f_counter_collection.csv")), counters(find(base, "w_counter_collection.csv"))
    fscale, wscale = COPY_BYTES / f["sr_copy_probe"][0], COPY_BYTES / w["sr_copy_probe"][0]

    def plan_of(run):
        """The dispatch plan of a counter run: its own bench line if its stdout was kept (the number of preconditioning
        launches depends on how fast the run is), else that of the traced run."""
        path = os.path.join(base, run + ".log")
        return bench_line(path)["detail"][wl]["dispatch_plan"] if os.path.exists(path) else plan

    plan_f, plan_w = plan_of("fetch"), plan_of("write")
    lead_f, lead_w = leading(plan_f, warmup), leading(plan_w, warmup)
    f_p, w_p = split_by_plan(f["sr_partial"], plan_f), split_by_plan(w["sr_partial"], plan_w)
    f_c, w_c = split_by_plan(f["sr_combine"], plan_f), split_by_plan(w["sr_combine"], plan_w)
    lead = leading(plan, warmup)
    out += ["", "## per mode: partial kernel (mean over the mode's dispatches, those in front of the first timed step left out: "
            "device preconditioning and %d warm-up steps)" % warmup, "",
            "Durations from the kernel trace (dispatch begin to end, the interval bench.py's HIP events attached to the launch "
            "measure when no profiler runs; under the profiler those events read about 10 us more and are not shown).  The gap is "
            "between the trace's end of the partial kernel and begin of the merge kernel.  Bytes: FETCH_SIZE / "
            "WRITE_SIZE per dispatch scaled by the copy kernel (1 GiB read, 1 GiB written: FETCH_SIZE = %.0f, WRITE_SIZE = %.0f, so one "
            "unit = %.1f B and %.1f B)." % (f["sr_copy_probe"][0], w["sr_copy_probe"][0], fscale, wscale), "",
            "| mode | skip | trace us (mean / min) | algorithmic MB | fetched MB | written MB | traffic / algorithmic | "
            "GB/s on trace mean | of 8 TB/s | merge kernel us | gap partial->merge us |", "|---|---|---|---|---|---|---|---|---|---|---|"]

    def mean(v):
        return sum(v) / max(len(v), 1)

    record = {}
    for label in [e[0] for e in plan]:
        m = det[label]
        k = lead[label]
        d = by_p[label][k:]
        kf, kw = lead_f[label], lead_w[label]
        fb, wb = mean(f_p[label][kf:]) * fscale, mean(w_p[label][kw:]) * wscale
        ab = m["algorithmic_bytes"]
        out.append("| %s | %.3f | %.1f / %.1f | %.2f | %.2f | %.2f | %.4f | %.0f | %.1f %% | %.1f | %.2f |" % (
            label, m["skip_ratio"], mean(d), min(d), ab / 1e6, fb / 1e6, wb / 1e6, (fb + wb) / ab,
            ab / mean(d) / 1e3, ab / mean(d) / 1e3 / 80.0, mean(by_c[label][k:]), mean(by_g[label][k:])))
        record[label] = {"kernel": "sr_partial_balanced_kernel", "fetch_bytes": round(fb), "write_bytes": round(wb),
                         "algorithmic_bytes": ab, "trace_us_mean": round(mean(d), 2), "trace_us_min": round(min(d), 2),
                         "merge_fetch_bytes": round(mean(f_c[label][kf:]) * fscale),
                         "merge_write_bytes": round(mean(w_c[label][kw:]) * wscale),
                         "merge_trace_us_mean": round(mean(by_c[label][k:]), 2),
                         "fetch_unit_bytes": round(fscale, 2), "write_unit_bytes": round(wscale, 2),
                         "kernel_source_sha": kernel_source_sha(), "command": cmd}
    out += ["", "Merge kernel traffic (fetched / written MB per dispatch): " +
            "; ".join("%s %.2f / %.2f" % (label, record[label]["merge_fetch_bytes"] / 1e6, record[label]["merge_write_bytes"] / 1e6)
                      for label in [e[0] for e in plan]) + ".", ""]
    out += utilisation_section(base, wl, "python3 $R/bench.py --workload %s --lean --steps 5 --warmup 2" % wl, det)
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    md = os.path.join(ROOT, "profiles", "sr_partial_balanced_kernel_%s.md" % wl)
    with open(md, "w") as fh:
        fh.write("\n".join(out))
    tj = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        allrec = json.load(open(tj))
    except (OSError, ValueError):
        allrec = {}
    allrec[wl] = record
    with open(tj, "w") as fh:
        json.dump(allrec, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("wrote", md, "and", tj)


if __name__ == "__main__":
    main(sys.argv)
