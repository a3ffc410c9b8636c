"""Turn rocprofv3 CSV output into the short text summaries kept next to the benchmarks.

  python profile_summary.py stats <..._kernel_stats.csv>
      per-kernel calls / average / share table of a `--kernel-trace --stats` run

  python profile_summary.py traffic --fetch <..._counter_collection.csv>
          --write <..._counter_collection.csv> --kernel fc_kernel --copy-bytes N
      HBM bytes per launch of one kernel from two `--pmc` runs (FETCH_SIZE, then WRITE_SIZE,
      both in KiB per dispatch), each scaled by what the same counter reads for the library's
      plain copy kernel moving N bytes in the same run.  Prints `key: value` lines; bench.py
      reads `traffic_bytes_per_launch` and `kernel_source_sha256` back.

  python profile_summary.py counters <..._counter_collection.csv> --kernel fc_big_walk_kernel
      mean of every collected counter per dispatch of one kernel

  python profile_summary.py split <..._kernel_trace.csv> --kernel fc_kernel
      average duration of one kernel in the benchmark's warm steps and in its cache-flushed steps
"""
import argparse
import csv
import os
import re
import sys

from bench import kernel_source_sha256      # the fingerprint bench.py checks stored counter summaries against


def short_name(name: str) -> str:
    """'_ZN2mt9fc_kernelIDF16bEEvNS_8GemmArgsE' or 'mt::fc_kernel<__bf16>(...)' -> a readable name."""
    m = re.match(r"_ZN2mt\d+([a-z_]+)I(DF16b|f)((?:L[ib]\d+E)*)", name)
    if m:
        args = ["bf16" if m.group(2) == "DF16b" else "float"] + re.findall(r"L[ib](\d+)E", m.group(3))
        return "mt::%s<%s>" % (m.group(1), ",".join(args))
    m = re.match(r"_ZN2mt\d+([a-z_]+)ILb([01])", name)
    if m:
        return "mt::%s<%s>" % (m.group(1), m.group(2))
    m = re.match(r"_ZN2mt\d+([a-z_]+)E", name)
    if m:
        return "mt::%s" % m.group(1)
    return re.sub(r"\(.*", "", name)


def stats(path: str, top: int = 12) -> str:
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    out = ["%-44s %8s %12s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "share%")]
    for r in rows[:top]:
        out.append("%-44s %8d %12.2f %10.2f %10.2f %7.2f" % (
            short_name(r["Name"])[:44], int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
            float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
    return "\n".join(out)


def split_warm_cold(trace_csv: str, kernel: str) -> str:
    """Average duration of one kernel's dispatches in a `--kernel-trace` run of bench.py, apart for the
    steps that ran right after the benchmark's cache flush (a large elementwise kernel in front of the
    step's segmentation kernel) and for all other steps."""
    rows = sorted(csv.DictReader(open(trace_csv)), key=lambda r: int(r["Start_Timestamp"]))
    flushed, step_cold = False, False
    acc = {False: [], True: []}
    for r in rows:
        name = r["Kernel_Name"]
        dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        if "elementwise_kernel" in name and dur > 100.0:
            flushed = True                       # the benchmark's 1 GiB rewrite in front of a step
        elif "batcher_kernel" in name:           # every step has exactly one
            step_cold, flushed = flushed, False
        elif kernel in short_name(name):
            acc[step_cold].append(dur)
    out = []
    for cold in (False, True):
        v = acc[cold]
        if v:
            out.append("%s %s: %d dispatches, avg %.2f us, min %.2f us, max %.2f us" % (
                kernel, "after a cache flush" if cold else "warm (steps back to back)", len(v), sum(v) / len(v), min(v), max(v)))
    return "\n".join(out)


def counter_means(path: str, counter: str) -> dict:
    """Mean counter value per dispatch, by readable kernel name."""
    acc = {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        s, n = acc.get(short_name(r["Kernel_Name"]), (0.0, 0))
        acc[short_name(r["Kernel_Name"])] = (s + float(r["Counter_Value"]), n + 1)
    return {k: (s / n, n) for k, (s, n) in acc.items()}


def pick(means: dict, needle: str):
    """The entry whose name contains `needle`; a trailing '*' pools every match (dispatch-weighted mean)."""
    pool = needle.endswith("*")
    hits = [k for k in means if needle.rstrip("*") in k]
    if not hits or (len(hits) != 1 and not pool):
        raise SystemExit("kernel %r matches %r" % (needle, hits))
    if not pool:
        return hits[0], means[hits[0]]
    n = sum(means[k][1] for k in hits)
    return " + ".join(sorted(hits)), (sum(means[k][0] * means[k][1] for k in hits) / n, n)


def traffic(fetch_csv: str, write_csv: str, kernel: str, copy_bytes: int) -> str:
    f, w = counter_means(fetch_csv, "FETCH_SIZE"), counter_means(write_csv, "WRITE_SIZE")
    (_, (cf, ncf)), (_, (cw, ncw)) = pick(f, "copy_kernel"), pick(w, "copy_kernel")
    (name, (kf, nkf)), (_, (kw, nkw)) = pick(f, kernel), pick(w, kernel)
    fetch_scale = copy_bytes / (cf * 1024.0)          # true bytes per counted byte
    write_scale = copy_bytes / (cw * 1024.0)
    fetch_b, write_b = kf * 1024.0 * fetch_scale, kw * 1024.0 * write_scale
    lines = [
        "kernel: %s" % name,
        "copy_kernel_bytes: %d" % copy_bytes,
        "copy_kernel_FETCH_SIZE_KiB: %.1f (%d dispatches)  -> scale %.3f" % (cf, ncf, fetch_scale),
        "copy_kernel_WRITE_SIZE_KiB: %.1f (%d dispatches)  -> scale %.3f" % (cw, ncw, write_scale),
        "kernel_FETCH_SIZE_KiB_per_launch: %.1f (%d dispatches)" % (kf, nkf),
        "kernel_WRITE_SIZE_KiB_per_launch: %.1f (%d dispatches)" % (kw, nkw),
        "fetch_bytes_per_launch: %.0f" % fetch_b,
        "write_bytes_per_launch: %.0f" % write_b,
        "traffic_bytes_per_launch: %.0f" % (fetch_b + write_b),
        "kernel_source_sha256: %s" % kernel_source_sha256(),
    ]
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("csv")
    s.add_argument("--top", type=int, default=12)
    t = sub.add_parser("traffic")
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    t.add_argument("--kernel", required=True)
    t.add_argument("--copy-bytes", type=int, required=True)
    w = sub.add_parser("split")
    w.add_argument("csv")
    w.add_argument("--kernel", required=True)
    c = sub.add_parser("counters")
    c.add_argument("csv")
    c.add_argument("--kernel", required=True)
    c.add_argument("--each", action="store_true", help="one line per kernel whose name contains --kernel")
    a = ap.parse_args(argv)
    if a.cmd == "stats":
        print(stats(a.csv, a.top))
    elif a.cmd == "split":
        print(split_warm_cold(a.csv, a.kernel))
    elif a.cmd == "traffic":
        print(traffic(a.fetch, a.write, a.kernel, a.copy_bytes))
    else:
        names = sorted({r["Counter_Name"] for r in csv.DictReader(open(a.csv))})
        for n in names:
            means = counter_means(a.csv, n)
            if a.each:
                for k in sorted(k for k in means if a.kernel in k):
                    print("%s %s: %.4g (mean of %d dispatches)" % (k, n, means[k][0], means[k][1]))
                continue
            k, (v, cnt) = pick(means, a.kernel)
            print("%s %s: %.4g (mean of %d dispatches)" % (k, n, v, cnt))


if __name__ == "__main__":
    main(sys.argv[1:])
