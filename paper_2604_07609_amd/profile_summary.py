"""Turns rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

  python -m paper_2604_07609_amd.profile_summary trace <kernel_trace.csv> <iterations.txt> <kernel> <workload> "<command>"
  python -m paper_2604_07609_amd.profile_summary pmc <fetch.csv> <write.csv> <iterations.txt> <kernel> <workload> "<cmd>"
  python -m paper_2604_07609_amd.profile_summary sq <counters.csv> <iterations.txt> <workload> "<command>"

`iterations.txt` is what `bench.py --dump-iterations` wrote in the same run: the kind of every iteration and the ordinal
of the scheduler kernel launch that ran it. The dispatches in the CSV are cut into chains at the scheduler kernel; the
n-th chain of the profile is the one whose scheduler launch has ordinal n, so every iteration finds its dispatches
whatever the launcher enqueued past the end of a window.
`trace`: per-kernel totals (what `--stats` prints) and the named kernel's average launch duration in the decode and in
the prefill iterations of the timed window. `pmc`: HBM bytes per launch of the named kernel in the timed decode
iterations from FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the same counter reads for the
64 MiB plain copy kernel that bench.py launches at its end. `sq`: the sequencers' wait and issue counters (SQ_WAVE_CYCLES,
SQ_WAIT_ANY, SQ_WAIT_INST_ANY, SQ_WAIT_INST_LDS, SQ_ACTIVE_INST_VALU, SQ_VALU_MFMA_BUSY_CYCLES, SQ_ACTIVE_INST_VMEM in
one --pmc run) per kernel and iteration kind, the MFMA share also relative to the register-only MFMA loop of the same run.
"""
import collections
import csv
import sys

COPY_BYTES = 64 << 20


def short(name):
    return name.split("(")[0]


def read_kinds(path):
    out = []
    for line in open(path):
        if line.startswith("#"):
            continue
        it, kind, n_seqs, n_tokens, ctx, timed, chain = (int(x) for x in line.split())
        out.append(dict(kind=kind, n_seqs=n_seqs, n_tokens=n_tokens, ctx_tokens=ctx, timed=timed, chain=chain))
    return out


def split_iterations(rows, value, order):
    """rows -> list of chains (lists of (kernel, value)) in launch order; a chain starts at k_sched."""
    rows = sorted(rows, key=order)
    its, cur = [], None
    for r in rows:
        n = short(r["Kernel_Name"])
        if n == "k_sched":
            cur = []
            its.append(cur)
        elif cur is not None and n.startswith("k_") and n not in ("k_copy_calibration", "k_mfma_calibration", "k_pack_weights", "k_rope_table", "k_open_window"):
            cur.append((n, value(r)))
    return its


def real_iterations(its, kinds):
    """The chains of the recorded iterations, in the order of `kinds`; [] when a chain is missing from the profile."""
    if any(k["chain"] >= len(its) for k in kinds):
        return []
    return [its[k["chain"]] for k in kinds]


def trace_summary(path, kinds_path, kernel, workload, command):
    rows = [r for r in csv.DictReader(open(path))]
    dur = collections.defaultdict(list)
    for r in rows:
        dur[short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in dur.values())
    out = ["# rocprofv3 --kernel-trace --stats: %s on %s" % (kernel, workload), "", "command: `%s`" % command, "",
           "| kernel | calls | total ms | avg us | % |", "|---|---|---|---|---|"]
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1]))[:14]:
        out.append("| %s | %d | %.1f | %.2f | %.1f |" % (k, len(v), sum(v) / 1e3, sum(v) / len(v), 100 * sum(v) / total))
    kinds = read_kinds(kinds_path)
    its = split_iterations(rows, lambda r: (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3,
                           lambda r: int(r["Start_Timestamp"]))
    its = real_iterations(its, kinds)
    out += ["", "iterations found in the trace by their scheduler launch: %d; iterations bench.py recorded: %d" % (len(its), len(kinds))]
    if len(its) == len(kinds):
        for label, kind in (("decode", 2), ("prefill", 1)):
            sel = [v for it, k in zip(its, kinds) if k["timed"] and k["kind"] == kind for n, v in it if n == kernel]
            if sel:
                out.append("%s, launches in the timed %s iterations: %d, average %.2f us" % (kernel, label, len(sel), sum(sel) / len(sel)))
        out.append("(bench.py measures the same launches with HIP events and reports them as roofline.avg_launch_us)")
        out += ["", "every kernel of the chain, average us per launch in the timed iterations (and launches per iteration):", "",
                "| kernel | decode | prefill |", "|---|---|---|"]
        names = []
        for it in its:
            for n, _ in it:
                if n not in names:
                    names.append(n)
        for nm in names:
            cells = []
            for kind in (2, 1):
                sel = [v for it, k in zip(its, kinds) if k["timed"] and k["kind"] == kind for n, v in it if n == nm]
                nit = sum(1 for k in kinds if k["timed"] and k["kind"] == kind)
                cells.append("%.2f (x%d)" % (sum(sel) / len(sel), round(len(sel) / max(1, nit))) if sel else "-")
            out.append("| %s | %s | %s |" % (nm, cells[0], cells[1]))
        for label, kind in (("decode", 2), ("prefill", 1)):
            tot = [sum(v for _, v in it) for it, k in zip(its, kinds) if k["timed"] and k["kind"] == kind]
            if tot:
                out.append("sum of kernel time per timed %s iteration: %.1f us on average" % (label, sum(tot) / len(tot)))
    else:
        out.append("(counts differ: no split by iteration kind)")
    return "\n".join(out) + "\n"


def sq_summary(path, kinds_path, workload, command):
    """Issue-side counters of the sequencers, per kernel and iteration kind, as shares of the wave cycles; the MFMA share is
    also given relative to the register-only MFMA loop bench.py runs at its end (the matrix cores' ceiling at this
    occupancy)."""
    names = ["SQ_WAIT_ANY", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_VALU", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_ACTIVE_INST_VMEM"]
    rows = [r for r in csv.DictReader(open(path))]
    disp = {}
    for r in rows:
        d = disp.setdefault(int(r["Dispatch_Id"]), {"Kernel_Name": r["Kernel_Name"], "Dispatch_Id": r["Dispatch_Id"]})
        d[r["Counter_Name"]] = float(r["Counter_Value"])
    ds = [disp[k] for k in sorted(disp)]
    ref = [d["SQ_VALU_MFMA_BUSY_CYCLES"] / d["SQ_WAVE_CYCLES"] for d in ds if short(d["Kernel_Name"]) == "k_mfma_calibration"]
    ref = sum(ref) / len(ref) if ref else None
    its, cur = [], None
    for d in ds:
        n = short(d["Kernel_Name"])
        if n == "k_sched":
            cur = []
            its.append(cur)
        elif cur is not None and n.startswith("k_") and n not in ("k_copy_calibration", "k_mfma_calibration", "k_pack_weights", "k_rope_table", "k_open_window"):
            cur.append((n, d))
    kinds = read_kinds(kinds_path)
    its = real_iterations(its, kinds)
    out = ["# rocprofv3 --pmc (SQ counters): where the waves of each kernel spend their cycles, %s" % workload, "", "command: `%s`" % command, "",
           "Shares of SQ_WAVE_CYCLES over the launches of the timed iterations. MFMA / loop = the MFMA share relative to the",
           "register-only MFMA loop of the same run (%s of its wave cycles): the matrix cores' utilisation over the kernel's time." % ("%.2f" % ref if ref else "n/a"), ""]
    if len(its) != len(kinds):
        return "\n".join(out + ["%d iterations with work in the counters, %d recorded by bench.py: no table" % (len(its), len(kinds))]) + "\n"
    out += ["| kernel | iterations | launches | wait (any) | wait (instruction) | wait (LDS) | VALU active | MFMA busy | MFMA / loop |", "|---|---|---|---|---|---|---|---|---|"]
    for kernel in ("k_qkv", "k_attention", "k_oproj", "k_gateup", "k_down", "k_lm_head"):
        for kind, label in ((1, "prefill"), (2, "decode")):
            tot, n = collections.Counter(), 0
            for it, k in zip(its, kinds):
                if k["timed"] and k["kind"] == kind:
                    for nm, d in it:
                        if nm == kernel:
                            n += 1
                            for c in names + ["SQ_WAVE_CYCLES"]:
                                tot[c] += d.get(c, 0.0)
            if n:
                wc = tot["SQ_WAVE_CYCLES"]
                out.append("| %s | %s | %d | %.2f | %.2f | %.2f | %.2f | %.2f | %s |" % (
                    kernel, label, n, tot["SQ_WAIT_ANY"] / wc, tot["SQ_WAIT_INST_ANY"] / wc, tot["SQ_WAIT_INST_LDS"] / wc,
                    tot["SQ_ACTIVE_INST_VALU"] / wc, tot["SQ_VALU_MFMA_BUSY_CYCLES"] / wc,
                    "%.2f" % (tot["SQ_VALU_MFMA_BUSY_CYCLES"] / wc / ref) if ref else "n/a"))
    return "\n".join(out) + "\n"


def pmc_summary(fetch_path, write_path, kinds_path, kernel, workload, command):
    out = ["# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: HBM traffic of %s on %s" % (kernel, workload), "",
           "commands (one counter per run): `%s`" % command, ""]
    kinds = read_kinds(kinds_path)
    tot = 0.0
    for label, path in (("FETCH_SIZE", fetch_path), ("WRITE_SIZE", write_path)):
        rows = [r for r in csv.DictReader(open(path))]
        # the first launch of the copy kernel is the 64 MiB one (the rate measurement after it copies 1 GiB per launch)
        copy = [float(r["Counter_Value"]) for r in sorted(rows, key=lambda r: int(r["Dispatch_Id"]))
                if short(r["Kernel_Name"]) == "k_copy_calibration"]
        factor = COPY_BYTES / 1024.0 / copy[0]
        its = split_iterations(rows, lambda r: float(r["Counter_Value"]), lambda r: int(r["Dispatch_Id"]))
        its = real_iterations(its, kinds)
        if len(its) != len(kinds):
            out.append("%s: %d iterations with work in the counters, %d recorded by bench.py: no traffic figure" % (label, len(its), len(kinds)))
            continue
        sel = [v for it, k in zip(its, kinds) if k["timed"] and k["kind"] == 2 for n, v in it if n == kernel]
        per = sum(sel) / len(sel) * 1024 * factor
        tot += per
        out.append("%s: copy kernel of %d KiB counts %.1f KiB -> scale %.4f; %s in the timed decode iterations: %d launches, mean %.1f KiB raw -> %.2f MB per launch"
                   % (label, COPY_BYTES // 1024, copy[0], factor, kernel, len(sel), sum(sel) / len(sel), per / 1e6))
    out += ["", "traffic_bytes_per_launch: %.0f" % tot]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "trace":
        sys.stdout.write(trace_summary(*sys.argv[2:7]))
    elif len(sys.argv) > 1 and sys.argv[1] == "pmc":
        sys.stdout.write(pmc_summary(*sys.argv[2:8]))
    elif len(sys.argv) > 1 and sys.argv[1] == "sq":
        sys.stdout.write(sq_summary(*sys.argv[2:6]))
    else:
        sys.exit(__doc__)
