"""Turn rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

    python -m paper_2410_11998_amd.rocprof_summary fused --kt DIR --fetch DIR --write DIR --out profiles/NAME.txt
                                                          [--traffic profiles/hbm_traffic.txt]
    python -m paper_2410_11998_amd.rocprof_summary counters --run LABEL=DIR[,DIR...] [--run ...] --out profiles/NAME.txt
    python -m paper_2410_11998_amd.rocprof_summary trace --run DIR [--run DIR ...] --out profiles/NAME.txt

Every DIR is the -d directory of ONE rocprofv3 run whose program was `python3 bench.py ...`, with the
program's output saved as DIR/bench.out (its JSON line is read from there):

* --kt     rocprofv3 --kernel-trace --stats --output-format csv        (kernel durations)
* --fetch  rocprofv3 --pmc FETCH_SIZE --output-format csv, bench.py --copy-calibration
* --write  rocprofv3 --pmc WRITE_SIZE --output-format csv, bench.py --copy-calibration
* --run    counters: rocprofv3 --pmc <any counters> --output-format csv (averaged per kernel; the hardware
           holds few counters at a time, so a label may take several runs of the same command);
           trace: rocprofv3 --kernel-trace --stats --output-format csv   (one section per run: the bench
           line's figures and the durations of the library's kernels)

The byte counters are scaled by what they read for the plain 1 GiB device copies bench.py
--copy-calibration runs last (the last four copy kernels of the run).  `fused` also rewrites the lines of
--traffic that belong to the workload: "workload kernel phase bytes source", which bench.py quotes
as roofline.traffic for exactly that kernel shape.

This is bookkeeping around the profiler's CSV files; nothing of the method is computed here.
"""

from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

PHASES = {0: "mix", 1: "updateonly", 2: "plain", 3: "loopstart", 4: "fold", 5: "alg1", 6: "mix_consensus"}


def parse_kernel(name: str):
    """(kernel shape as bench.py names it, phase name) of one of the library's kernels, else (None, None)."""
    m = re.search(r"\b(k_tile|k_direct|k_acc)<(.*)>\(", name)
    if not m:
        return None, None
    args = [a.strip().split("::")[-1] for a in m.group(2).split(",")]
    kind = m.group(1)
    try:
        if kind == "k_tile":          # <param type, grad type, phase, waves, vectors, non-temporal>
            return f"k_tile<{args[0]},{args[1]},{args[3]},{args[4]},{args[5]}>", PHASES[int(args[2])]
        if kind == "k_direct":        # <param type, grad type, phase, hints: 0 none, 1 all, 2 all but the sources'>
            hint = {"0": "false", "1": "true", "2": "shared"}.get(args[3], args[3])
            return f"k_direct<{args[0]},{args[1]},{hint}>", PHASES[int(args[2])]
        return f"k_acc<{args[0]},{args[1]},{args[3]}>", PHASES[int(args[2])]     # <grad type, elements per vector, phase, nt>
    except (IndexError, KeyError, ValueError):
        return None, None


def one_file(directory: str, pattern: str) -> str:
    hits = glob.glob(os.path.join(directory, "**", pattern), recursive=True)
    if not hits:
        raise SystemExit(f"no {pattern} under {directory}")
    return max(hits, key=os.path.getmtime)


def bench_line(directory: str) -> dict:
    with open(os.path.join(directory, "bench.out")) as f:
        lines = [l for l in f if l.startswith("{")]
    if not lines:
        raise SystemExit(f"no JSON line in {directory}/bench.out")
    return json.loads(lines[-1])


def bench_command(directory: str) -> str:
    """The bench.py command of a run, as rocprofv3 logged it."""
    with open(os.path.join(directory, "bench.out")) as f:
        for l in f:
            m = re.search(r"'(python3? \S*bench\.py[^']*)'", l)
            if m:
                return re.sub(r"\S*/bench\.py", "bench.py", m.group(1))
    return "python3 bench.py ..."


PROBE_SHAPE, PROBE_PHASE = "k_tile<TF32,TF32,4,2,true>", "mix"
PROBE_LABEL = "mix (arena probe)"


def probe_launches(directory: str) -> int:
    """How many mixing passes the arena's timing probe launched before the workload's own kernels (bench.py
    reports it); they are the first dispatches of that kernel shape and are listed apart."""
    return int(bench_line(directory)["config"].get("placement_probe_launches") or 0)


def library_dispatches(directory: str, pattern: str, name_col: str):
    """Rows of a per-dispatch CSV that belong to the library's kernels (or plain copies), in dispatch order,
    as (shape, phase, row), with the arena probe's launches relabelled."""
    left = probe_launches(directory)
    with open(one_file(directory, pattern)) as f:
        rows = sorted(csv.DictReader(f), key=lambda r: int(r["Dispatch_Id"]))
    probe_ids = set()
    for r in rows:
        shape, phase = parse_kernel(r[name_col])
        if shape is None and "copyBuffer" in r[name_col]:
            shape, phase = "copy", ""
        if shape is None:
            continue
        if (shape, phase) == (PROBE_SHAPE, PROBE_PHASE) and (r["Dispatch_Id"] in probe_ids or left > 0):
            if r["Dispatch_Id"] not in probe_ids:       # a counter file has one row per counter and dispatch
                probe_ids.add(r["Dispatch_Id"])
                left -= 1
            phase = PROBE_LABEL
        yield shape, phase, r


def kernel_stats(directory: str):
    """(shape, phase, calls, avg ms, min ms, max ms) from the per-dispatch kernel trace."""
    ns = collections.defaultdict(list)
    for shape, phase, r in library_dispatches(directory, "*kernel_trace.csv", "Kernel_Name"):
        if shape != "copy":
            ns[(shape, phase)].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return sorted((shape, phase, len(v), mean(v) / 1e6, min(v) / 1e6, max(v) / 1e6) for (shape, phase), v in ns.items())


def counter_values(directory: str):
    """{(kernel shape or 'copy', phase): {counter: [values per dispatch]}}"""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for shape, phase, r in library_dispatches(directory, "*counter_collection.csv", "Kernel_Name"):
        out[(shape, phase)][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return out


def mean(v):
    return sum(v) / len(v)


def cmd_fused(a) -> int:
    j = bench_line(a.kt)
    wl = j["config"]["workload"]
    lines = [f"rocprofv3 summary: {j['config']['path']} step, workload {wl}, one MI355X", "",
             "Commands (run from /tmp with TMPDIR=/tmp; paths relative to the repository root; written by",
             "python -m paper_2410_11998_amd.rocprof_summary fused from the profiler's CSV files):",
             f"  rocprofv3 --kernel-trace --stats --output-format csv -d OUT/kt -- {bench_command(a.kt)}",
             f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -- {bench_command(a.fetch)}",
             f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -- {bench_command(a.write)}", "",
             "bench.py line of the kernel-trace run (per_config / packed / cpu_baseline left out):",
             "  " + json.dumps({k: v for k, v in j.items() if k not in ("per_config", "packed", "cpu_baseline")}), "",
             "Kernel statistics (from *_kernel_trace.csv, per dispatch), the library's kernels; shape = <param type, grad type,",
             "[waves, vectors per lane,] non-temporal>; the arena's timing probe launches the 16-source mixing kernel on 2 GiB:",
             f"  {'kernel':34s} {'phase':17s} {'calls':>5s} {'avg ms':>9s} {'min ms':>9s} {'max ms':>9s}"]
    for shape, phase, calls, avg, lo, hi in kernel_stats(a.kt):
        lines.append(f"  {shape:34s} {phase:17s} {calls:5d} {avg:9.3f} {lo:9.3f} {hi:9.3f}")
    fetch, write = counter_values(a.fetch), counter_values(a.write)
    cal_f = mean(fetch[("copy", "")]["FETCH_SIZE"][-4:])
    cal_w = mean(write[("copy", "")]["WRITE_SIZE"][-4:])
    kf, kw = 1048576.0 / cal_f, 1048576.0 / cal_w
    lines += ["", "HBM traffic per dispatch (KiB as the counters report them):",
              f"  calibration: plain device copies of 1 GiB (1048576 KiB read, 1048576 KiB written; the last four copy kernels",
              f"  of the run, averaged): FETCH_SIZE reads {cal_f:.0f}, WRITE_SIZE reads {cal_w:.0f}",
              f"  => scale factors: FETCH_SIZE x {kf:.4f}, WRITE_SIZE x {kw:.4f}"]
    traffic = []
    R, d = j["config"]["n_rows"], j["config"]["d"]
    for key in sorted(k for k in fetch if k[0] != "copy"):
        fv, wv = fetch[key]["FETCH_SIZE"], write.get(key, {}).get("WRITE_SIZE", [0.0])
        fb, wb = mean(fv) * kf * 1024, mean(wv) * kw * 1024
        lines.append(f"  {key[0]:34s} {key[1]:17s} dispatches {len(fv):3d}  FETCH_SIZE avg {mean(fv):12.0f} -> {fb / 1e9:7.2f} GB   "
                     f"WRITE_SIZE avg {mean(wv):12.0f} -> {wb / 1e9:7.2f} GB   total {(fb + wb) / 1e9:7.2f} GB"
                     + ("" if key[1] == PROBE_LABEL else f" = {(fb + wb) / (R * d):.3f} B per replica-param"))
        if key[1] != PROBE_LABEL:
            traffic.append((wl, key[0], key[1], fb + wb))
    ro = j["roofline"]
    lines += ["", f"Algorithmic bytes per dispatch, average over the timed steps (R*d = {R * d} elements): {ro['algorithmic_bytes_per_launch']:.0f}",
              f"roofline of the kernel-trace run: achieved {ro['achieved']:.0f} GB/s of {ro['peak']:.0f} GB/s = {ro['frac']:.3f}; "
              f"avg launch {ro['avg_launch_ms']:.3f} ms; by phase {json.dumps(ro['ms_by_phase'])}"]
    with open(a.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    if a.traffic:
        keep = []
        if os.path.exists(a.traffic):
            with open(a.traffic) as f:
                keep = [l.rstrip("\n") for l in f if l.strip() and not l.startswith("#") and l.split()[0] != wl]
        head = ["# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by a plain 1 GiB copy),",
                "# written by python -m paper_2410_11998_amd.rocprof_summary fused; bench.py quotes them as roofline.traffic.",
                "# workload kernel phase bytes source"]
        rows = keep + [f"{w} {k} {p} {b:.0f} {os.path.relpath(a.out, os.path.dirname(os.path.dirname(os.path.abspath(a.traffic))))}"
                       for w, k, p, b in traffic]
        with open(a.traffic, "w") as f:
            f.write("\n".join(head + sorted(rows)) + "\n")
    print("\n".join(lines))
    return 0


def cmd_counters(a) -> int:
    lines = ["rocprofv3 counter summary (averages per dispatch of the library's kernels), one MI355X", "",
             "Runs (from /tmp with TMPDIR=/tmp; written by python -m paper_2410_11998_amd.rocprof_summary counters):"]
    table = collections.defaultdict(dict)      # (kernel, phase, counter) -> {label: value}
    labels = []
    for spec in a.run:
        label, directories = spec.split("=", 1)
        labels.append(label)
        for directory in directories.split(","):
            vals = counter_values(directory)
            names = sorted({c for v in vals.values() for c in v})
            j = bench_line(directory)
            lines.append(f"  {label}: rocprofv3 --pmc {' '.join(names)} --output-format csv -d OUT -- {bench_command(directory)}")
            lines.append(f"      {j['config']['workload']}, {j['config']['hbm_layout']}: {j['ms_per_step']:.3f} ms per step, "
                         f"roofline fraction {j['roofline']['frac']:.3f}")
            for (shape, phase), cs in vals.items():
                if shape == "copy" or phase == PROBE_LABEL:
                    continue
                for c, v in cs.items():
                    table[(shape, phase, c)][label] = mean(v)
    lines += ["", f"  {'kernel':30s} {'phase':10s} {'counter':44s} " + " ".join(f"{l:>14s}" for l in labels)]
    for (shape, phase, c) in sorted(table):
        row = table[(shape, phase, c)]
        lines.append(f"  {shape:30s} {phase:10s} {c:44s} " + " ".join(f"{row[l]:14.5g}" if l in row else f"{'-':>14s}" for l in labels))
    derived = [("mean read latency at the L2-to-memory interface, L2 cycles", "TCC_EA0_RDREQ_LEVEL_sum", "TCC_EA0_RDREQ_sum"),
               ("mean write latency at the L2-to-memory interface, L2 cycles", "TCC_EA0_WRREQ_LEVEL_sum", "TCC_EA0_WRREQ_sum"),
               ("reads in flight per L2 channel (level / channel-cycles)", "TCC_EA0_RDREQ_LEVEL_sum", "TCC_CYCLE_sum"),
               ("read credit stalls, share of L2 channel-cycles", "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum", "TCC_CYCLE_sum"),
               ("write credit stalls, share of L2 channel-cycles", "TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum", "TCC_CYCLE_sum"),
               ("L2 tag stalls, share of L2 channel-cycles", "TCC_TAG_STALL_sum", "TCC_CYCLE_sum"),
               ("mean read latency seen from the L1, cycles", "TCP_TCC_READ_REQ_LATENCY_sum", "TCP_TCC_READ_REQ_sum"),
               ("mean write latency seen from the L1, cycles", "TCP_TCC_WRITE_REQ_LATENCY_sum", "TCP_TCC_WRITE_REQ_sum"),
               ("L1 address-translation miss rate", "TCP_UTCL1_TRANSLATION_MISS_sum", "TCP_UTCL1_REQUEST_sum"),
               ("wavefront cycles waiting on any instruction, share", "SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES")]
    keys = sorted({(shape, phase) for (shape, phase, _c) in table})
    lines += ["", "Derived (ratio of two counters above):",
              f"  {'kernel':30s} {'phase':10s} {'quantity':62s} " + " ".join(f"{l:>14s}" for l in labels)]
    for shape, phase in keys:
        for text, num, den in derived:
            n_, d_ = table.get((shape, phase, num)), table.get((shape, phase, den))
            if n_ and d_:
                lines.append(f"  {shape:30s} {phase:10s} {text:62s} " +
                             " ".join(f"{n_[l] / d_[l]:14.5g}" if l in n_ and l in d_ and d_[l] else f"{'-':>14s}" for l in labels))
    with open(a.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


def cmd_trace(a) -> int:
    lines = ["rocprofv3 kernel-trace summary of further bench.py runs (other entry points and call sequences), one MI355X", "",
             "Each section: rocprofv3 --kernel-trace --stats --output-format csv -d OUT -- <command> (from /tmp with TMPDIR=/tmp;",
             "written by python -m paper_2410_11998_amd.rocprof_summary trace).  Calls include warm-up steps and every timed region.",
             "Kernel shape = <param type, grad type, [waves, vectors per lane,] non-temporal>.  \"mix (arena probe)\": the 16-source",
             "mixing passes over 2 GiB with which the arena finds the thirds of the memory before the workload is set up."]
    for directory in a.run:
        j = bench_line(directory)
        ro, c = j["roofline"], j["config"]
        lines += ["", f"{bench_command(directory)}",
                  f"  {c['workload']}, path {c['path']}, {c['launches_per_step']} launch(es) per step"
                  + (f" on {c['bucket_streams']} stream(s)" if c.get("bucket_streams") else "")
                  + f": {j['ms_per_step']:.3f} ms per step, {j['value']:.4g} replica-params/s, "
                  f"{ro['achieved']:.0f} GB/s = {ro['frac']:.3f} of peak on the bytes this path moves; host {j.get('host_us_per_call') or 0:.1f} us per call",
                  f"  {'kernel':34s} {'phase':17s} {'calls':>6s} {'avg ms':>9s} {'min ms':>9s} {'max ms':>9s}"]
        for shape, phase, calls, avg, lo, hi in kernel_stats(directory):
            lines.append(f"  {shape:34s} {phase:17s} {calls:6d} {avg:9.3f} {lo:9.3f} {hi:9.3f}")
    with open(a.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    f = sub.add_parser("fused")
    for name in ("--kt", "--fetch", "--write", "--out"):
        f.add_argument(name, required=True)
    f.add_argument("--traffic", default=None)
    c = sub.add_parser("counters")
    c.add_argument("--run", action="append", required=True, metavar="LABEL=DIR")
    c.add_argument("--out", required=True)
    t = sub.add_parser("trace")
    t.add_argument("--run", action="append", required=True, metavar="DIR")
    t.add_argument("--out", required=True)
    a = ap.parse_args()
    return {"fused": cmd_fused, "counters": cmd_counters, "trace": cmd_trace}[a.cmd](a)


if __name__ == "__main__":
    sys.exit(main())
