"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

Two kinds of input, each the output directory (-d) of one rocprofv3 run of bench.py:

  kernel trace   rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -- python3 bench.py ...
                 -> per kernel: calls, and median / min / mean / max duration of the TIMED calls only.  The calls that
                 belong to bench.py's warm-up steps are dropped: a kernel launched k times per step has its first
                 k * warmup calls discarded.  A kernel launched several times per step (one launch per direction, say)
                 is also reported per position within the step.
  counters       rocprofv3 --pmc <counters> --output-format csv -d <dir> -- python3 bench.py ...
                 -> per kernel and counter: mean value per dispatch.  FETCH_SIZE / WRITE_SIZE (KiB) are turned into
                 bytes with the scale a plain 1 GiB device copy gives (the --calibration directories:
                 runs of `bench.py --calibrate-copy` under the same counter).

Usage:
  python -m paper_2511_15927_amd.profile_summary stats <dir> --warmup 5 --steps 20 [--command "..."] [-o out.txt]
  python -m paper_2511_15927_amd.profile_summary pmc <dir> [<dir> ...] [--calibration-fetch <dir>] [--calibration-write <dir>]
         [--kernel <substring>] [--command "..."] [-o out.txt]

Nothing here touches the GPU; the summaries hold the command that produced their input.
"""
import argparse
import collections
import csv
import glob
import os
import statistics
import sys


def _rows(directory, suffix):
    files = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not files:
        raise SystemExit("no *%s under %s" % (suffix, directory))
    for f in files:
        with open(f, newline="") as fh:
            for r in csv.DictReader(fh):
                yield r


def kernel_durations(directory):
    """{kernel name: [duration_ns of every dispatch, in dispatch order]}"""
    rows = sorted(_rows(directory, "_kernel_trace.csv"), key=lambda r: int(r["Start_Timestamp"]))
    out = collections.OrderedDict()
    for r in rows:
        out.setdefault(r["Kernel_Name"], []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return out


def summarise_stats(directory, warmup, steps, command=None):
    lines = ["rocprofv3 kernel trace, per-kernel durations of the timed steps (one MI355X)"]
    if command:
        lines.append("command (from /tmp, TMPDIR=/tmp): " + command)
    lines.append("warm-up steps dropped: %d; timed steps: %d" % (warmup, steps))
    lines.append("")
    lines.append("%-78s %6s %8s %12s %12s %12s %12s" % ("kernel [launch within the step]", "calls", "timed", "median_ns",
                                                        "min_ns", "mean_ns", "max_ns"))
    total = warmup + steps
    for name, durs in kernel_durations(directory).items():
        per_step = len(durs) // total if total and len(durs) % total == 0 else 0
        timed = durs[per_step * warmup:] if per_step else durs
        note = "" if per_step else "  (calls not a multiple of the steps: nothing dropped)"
        lines.append("%-78s %6d %8d %12.0f %12d %12.0f %12d%s" % (name[:78], len(durs), len(timed), statistics.median(timed),
                                                                 min(timed), statistics.fmean(timed), max(timed), note))
        if per_step > 1:
            for k in range(per_step):
                part = timed[k::per_step]
                lines.append("%-78s %6s %8d %12.0f %12d %12.0f %12d" % ("    launch %d of %d in a step" % (k + 1, per_step), "",
                                                                       len(part), statistics.median(part), min(part),
                                                                       statistics.fmean(part), max(part)))
    return "\n".join(lines) + "\n"


_counters_per_dispatch = {}


def counter_means(directory, kernel_filter=None):
    """{(kernel, counter): (mean per dispatch, dispatches)}; also the launch geometry of each kernel."""
    agg = collections.defaultdict(lambda: [0.0, 0])
    geom = {}
    rows = list(_rows(directory, "_counter_collection.csv"))
    per = collections.defaultdict(set)
    for r in rows:
        per[r["Kernel_Name"]].add(r["Counter_Name"])
    _counters_per_dispatch.clear()
    _counters_per_dispatch.update({k: len(v) for k, v in per.items()})
    for r in rows:
        k = r["Kernel_Name"]
        if kernel_filter and kernel_filter not in k:
            continue
        a = agg[(k, r["Counter_Name"])]
        a[0] += float(r["Counter_Value"])
        a[1] += 1
        if "Start_Timestamp" in r:   # the dispatch's own duration (under counter collection: an upper bound)
            t = agg[(k, "DURATION_NS_UNDER_PMC")]
            t[0] += (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / max(1, _counters_per_dispatch.get(k, 1))
            t[1] += 1.0 / max(1, _counters_per_dispatch.get(k, 1))
        if k not in geom and "Grid_Size" in r:
            geom[k] = (int(r["Grid_Size"]), int(r["Workgroup_Size"]))
    return {k: (v[0] / v[1], v[1]) for k, v in agg.items()}, geom


def _copy_scale(directory, counter):
    """Bytes per KiB-count of `counter`, from a run of `bench.py --calibrate-copy` (1 GiB read and written per copy)."""
    means, _ = counter_means(directory)
    vals = [v[0] for (k, c), v in means.items() if c == counter and "copy" in k.lower()]
    if not vals:
        return None, None
    kib = max(vals)
    return (1 << 30) / (kib * 1024.0), kib


def summarise_pmc(directories, kernel_filter=None, cal_fetch=None, cal_write=None, command=None):
    lines = ["# rocprofv3 hardware counters, mean per dispatch (one MI355X)"]
    if command:
        lines.append("# command (from /tmp, TMPDIR=/tmp), one counter set per run: " + command)
    merged, geoms = {}, {}
    for d in directories:
        m, g = counter_means(d, kernel_filter)
        merged.update(m)
        geoms.update(g)
    kernels = sorted({k for k, _ in merged})
    scales = {}
    for counter, d in (("FETCH_SIZE", cal_fetch), ("WRITE_SIZE", cal_write)):
        if d:
            scale, kib = _copy_scale(d, counter)
            if scale:
                scales[counter] = scale
                lines.append("COPY_1GIB_%s_KIB=%g" % (counter, kib))
                lines.append("%s_SCALE=%.4f" % (counter.split("_")[0], scale))
    for k in kernels:
        lines.append("# kernel: " + k)
        if k in geoms:
            lines.append("GRID_THREADS=%d" % geoms[k][0])
            lines.append("WORKGROUP_THREADS=%d" % geoms[k][1])
        for (kk, c), (mean, n) in sorted(merged.items()):
            if kk != k:
                continue
            lines.append("%s=%g" % (c + ("_KIB" if c in ("FETCH_SIZE", "WRITE_SIZE") else ""), mean))
            if c in scales:
                lines.append("%s_BYTES_PER_LAUNCH=%g" % (c.split("_")[0], mean * 1024.0 * scales[c]))
    return "\n".join(lines) + "\n"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("directory")
    s.add_argument("--warmup", type=int, default=5)
    s.add_argument("--steps", type=int, default=20)
    s.add_argument("--command")
    s.add_argument("-o", "--output")
    p = sub.add_parser("pmc")
    p.add_argument("directories", nargs="+")
    p.add_argument("--kernel")
    p.add_argument("--calibration-fetch")
    p.add_argument("--calibration-write")
    p.add_argument("--command")
    p.add_argument("-o", "--output")
    a = ap.parse_args(argv)
    if a.what == "stats":
        text = summarise_stats(a.directory, a.warmup, a.steps, a.command)
    else:
        text = summarise_pmc(a.directories, a.kernel, a.calibration_fetch, a.calibration_write, a.command)
    if a.output:
        with open(a.output, "w") as fh:
            fh.write(text)
    sys.stdout.write(text)


if __name__ == "__main__":
    main()
