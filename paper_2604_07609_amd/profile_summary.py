"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

  python -m paper_2604_07609_amd.profile_summary trace  <kernel_trace.csv> <kernel> <workload> "<command>"
  python -m paper_2604_07609_amd.profile_summary pmc    <fetch_counter.csv> <write_counter.csv> <kernel> <workload> "<cmd>"

`trace`: per-kernel totals (what `--stats` prints) and, for the named kernel, the average duration of its launches
split into the decode class (launches within 1.35x of the median: one weight-streaming pass) and the rest (prefill).
`pmc`: HBM bytes per launch of the named kernel from FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by
what the same counter reads for the 64 MiB plain copy kernel that bench.py launches at its end.
"""
import collections
import csv
import statistics
import sys

COPY_BYTES = 64 << 20


def short(name):
    return name.split("(")[0]


def trace_summary(path, kernel, workload, command):
    rows = [r for r in csv.DictReader(open(path))]
    dur = collections.defaultdict(list)
    for r in rows:
        dur[short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in dur.values())
    out = ["# rocprofv3 --kernel-trace --stats: %s on %s" % (kernel, workload), "", "command: `%s`" % command, "",
           "| kernel | calls | total ms | avg us | % |", "|---|---|---|---|---|"]
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1]))[:14]:
        out.append("| %s | %d | %.1f | %.2f | %.1f |" % (k, len(v), sum(v) / 1e3, sum(v) / len(v), 100 * sum(v) / total))
    v = [x for x in dur[kernel] if x > 8.0]          # launches of iterations past the end of a window do nothing
    med = statistics.median(v)
    dec = [x for x in v if x <= 1.35 * med]
    pre = [x for x in v if x > 1.35 * med]
    out += ["", "%s, launches that do work: %d, average %.2f us" % (kernel, len(v), sum(v) / len(v)),
            "  decode class (<= 1.35 x median %.2f us): %d launches, average %.2f us" % (med, len(dec), sum(dec) / len(dec))]
    if pre:
        out.append("  prefill class: %d launches, average %.2f us" % (len(pre), sum(pre) / len(pre)))
    out.append("  (bench.py reports the same two classes over its timed iterations only; warm-up launches are included here)")
    return "\n".join(out) + "\n"


def counter(path, kernel):
    vals, copy = [], []
    for r in csv.DictReader(open(path)):
        n = short(r["Kernel_Name"])
        if n == kernel:
            vals.append(float(r["Counter_Value"]))
        elif n == "k_copy_calibration":
            copy.append(float(r["Counter_Value"]))
    return vals, copy


def pmc_summary(fetch_path, write_path, kernel, workload, command):
    out = ["# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: HBM traffic of %s on %s" % (kernel, workload), "",
           "commands (one counter per run): `%s`" % command, ""]
    tot = 0.0
    for label, path, copied in (("FETCH_SIZE", fetch_path, COPY_BYTES), ("WRITE_SIZE", write_path, COPY_BYTES)):
        vals, copy = counter(path, kernel)
        vals = [x for x in vals if x > 16.0]
        med = statistics.median(vals)
        dec = [x for x in vals if x <= 1.35 * med] if label == "FETCH_SIZE" else vals
        factor = copied / 1024.0 / copy[0]
        if label == "WRITE_SIZE":           # classify by the fetch classes is not possible across runs: use the median
            per = med * 1024 * factor
        else:
            per = sum(dec) / len(dec) * 1024 * factor
        tot += per
        out.append("%s: copy kernel of %d KiB reads %.1f KiB -> scale %.4f; %s decode class %s = %.1f KiB raw -> %.2f MB per launch"
                   % (label, copied // 1024, copy[0], factor, kernel, "mean" if label == "FETCH_SIZE" else "median",
                      per / 1024 / factor, per / 1e6))
    out += ["", "traffic_bytes_per_launch: %.0f" % tot]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if sys.argv[1] == "trace":
        sys.stdout.write(trace_summary(*sys.argv[2:6]))
    elif sys.argv[1] == "pmc":
        sys.stdout.write(pmc_summary(*sys.argv[2:7]))
    else:
        sys.exit(__doc__)
