"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2212_05271_amd.profile_summary trace  KERNEL_STATS.csv --title T --command C --out profiles/X.md
    python -m paper_2212_05271_amd.profile_summary traffic --fetch F.csv --write W.csv --cal-fetch CF.csv --cal-write CW.csv
                                                   --kernel em_whole_small --title T --command C --out profiles/X.md

`trace` takes the kernel_stats.csv of `rocprofv3 --kernel-trace --stats` and writes one table row per kernel
(calls, average, total, share).  `traffic` takes the counter_collection.csv files of two `rocprofv3 --pmc` runs
(FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) of the same command and of the copy calibration
(`bench.py --copy-calibration`: 256 MiB device-to-device copies of known size), scales each counter by what it
reads for the copy, and writes the bytes per launch of the kernels whose name contains --kernel.  bench.py reads
the line "bytes per launch" of profiles/em_pass_hbm_traffic.md.

    python -m paper_2212_05271_amd.profile_summary counters COUNTERS.csv [MORE.csv ...] --title T --command C --out profiles/X.md

`counters` writes the mean per launch of every counter in the given counter_collection.csv files, one row per
kernel.  When the read-request counters TCC_EA0_RDREQ_32B/64B/128B_sum are among them it adds the bytes they
stand for (32, 64 and 128 bytes per request), and with WRITE_SIZE (KiB) the bytes written.
"""

from __future__ import annotations

import argparse
import collections
import csv
import re


def short_name(n):
    if "at::native" in n:
        return "torch elementwise (fills, copies)"
    n = n.replace("void ", "").replace("(anonymous namespace)::", "")
    m = re.match(r"([A-Za-z_0-9]+(<[^>]*>)?)", n)
    return m.group(1) if m else n[:48]


def trace(a):
    rows = list(csv.DictReader(open(a.stats)))
    out = [f"# {a.title}\n", "Command (run from /tmp with TMPDIR=/tmp, repository root as working directory):\n",
           f"    {a.command}\n"]
    if a.note:
        out.append(a.note + "\n")
    out.append("| kernel | calls | average (us) | total (ms) | share |\n|---|---:|---:|---:|---:|")
    tot = 0.0
    for r in rows:
        if "rocclr" in r["Name"]:
            continue
        tot += float(r["TotalDurationNs"])
        out.append("| %s | %s | %.2f | %.3f | %.2f %% |" % (short_name(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                                                        float(r["TotalDurationNs"]) / 1e6, float(r["Percentage"])))
    out.append("\nSum over all kernels: %.2f ms." % (tot / 1e6))
    open(a.out, "w").write("\n".join(out) + "\n")


def _counter(fn, name):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(fn)):
        if r["Counter_Name"] == name:
            per[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per


def traffic(a):
    fetch, write = _counter(a.fetch, "FETCH_SIZE"), _counter(a.write, "WRITE_SIZE")
    calf, calw = _counter(a.cal_fetch, "FETCH_SIZE"), _counter(a.cal_write, "WRITE_SIZE")

    def copy_mean(per):
        vals = [v for k, vs in per.items() if "copy" in k.lower() for v in vs if v > 1000.0]
        return sum(vals) / len(vals)

    copy_kib = 256.0 * 1024.0
    kf, kw = copy_kib / copy_mean(calf), copy_kib / copy_mean(calw)
    out = [f"# {a.title}\n", "Commands (run from /tmp with TMPDIR=/tmp, repository root as working directory), one counter per run:\n",
           f"    rocprofv3 --pmc FETCH_SIZE ... -- {a.command}", f"    rocprofv3 --pmc WRITE_SIZE ... -- {a.command}",
           "    rocprofv3 --pmc FETCH_SIZE ... -- python3 bench.py --copy-calibration",
           "    rocprofv3 --pmc WRITE_SIZE ... -- python3 bench.py --copy-calibration\n",
           "The counters are in KiB per dispatch.  For the 256 MiB device-to-device copy they read %.0f (FETCH_SIZE) and "
           "%.0f (WRITE_SIZE) KiB, so they are scaled by %.3f and %.3f.\n" % (copy_mean(calf), copy_mean(calw), kf, kw),
           "| kernel | launches | read per launch (MB) | written per launch (MB) |\n|---|---:|---:|---:|"]
    dom = None
    for k in sorted(fetch, key=lambda k: -sum(fetch[k])):
        if "rocclr" in k or "at::native" in k:
            continue
        f = sum(fetch[k]) / len(fetch[k]) * kf * 1024.0
        w = sum(write.get(k, [0.0])) / max(len(write.get(k, [0.0])), 1) * kw * 1024.0
        out.append("| %s | %d | %.2f | %.2f |" % (short_name(k), len(fetch[k]), f / 1e6, w / 1e6))
        if a.kernel in k and dom is None:
            dom = (short_name(k), len(fetch[k]), f, w)
    if dom:
        out.append("\nDominant kernel %s, %d launches in the run:" % (dom[0], dom[1]))
        out.append("bytes per launch (FETCH_SIZE + WRITE_SIZE, calibrated): %d" % round(dom[2] + dom[3]))
        if a.algorithmic_bytes:
            out.append("algorithmic bytes per launch: %d (%s)" % (a.algorithmic_bytes, a.algorithmic_note))
            out.append("ratio: %.2f" % ((dom[2] + dom[3]) / a.algorithmic_bytes))
    open(a.out, "w").write("\n".join(out) + "\n")


def counters(a):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for fn in a.files:
        for r in csv.DictReader(open(fn)):
            per[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = []
    for k in per:
        for c in per[k]:
            if c not in names:
                names.append(c)
    sizes = {"TCC_EA0_RDREQ_32B_sum": 32, "TCC_EA0_RDREQ_64B_sum": 64, "TCC_EA0_RDREQ_128B_sum": 128}
    with_bytes = all(s in names for s in sizes)
    head = ["kernel", "launches"] + names + (["read per launch (MB)"] if with_bytes else []) + \
           (["written per launch (MB)"] if "WRITE_SIZE" in names else [])
    out = [f"# {a.title}\n", "Commands (run from /tmp with TMPDIR=/tmp, repository root as working directory):\n"]
    out += ["    " + c for c in a.command]
    if a.note:
        out.append("\n" + a.note)
    out.append("\nMean per launch.\n")
    out.append("| " + " | ".join(head) + " |")
    out.append("|---|" + "---:|" * (len(head) - 1))
    for k in sorted(per, key=lambda k: -sum(sum(v) for v in per[k].values())):
        if "rocclr" in k and not a.keep_copies:
            continue
        if "at::native" in k:
            continue
        mean = {c: sum(v) / len(v) for c, v in per[k].items()}
        n = max(len(v) for v in per[k].values())
        row = [short_name(k) if "rocclr" not in k else k, str(n)] + ["%.4g" % mean[c] if c in mean else "" for c in names]
        if with_bytes:
            row.append("%.2f" % (sum(mean.get(c, 0.0) * b for c, b in sizes.items()) / 1e6))
        if "WRITE_SIZE" in names:
            row.append("%.2f" % (mean.get("WRITE_SIZE", 0.0) * 1024.0 / 1e6))
        out.append("| " + " | ".join(row) + " |")
    open(a.out, "w").write("\n".join(out) + "\n")


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("stats")
    t.add_argument("--title", required=True)
    t.add_argument("--command", required=True)
    t.add_argument("--note", default="")
    t.add_argument("--out", required=True)
    f = sub.add_parser("traffic")
    for n in ("fetch", "write", "cal-fetch", "cal-write"):
        f.add_argument("--" + n, required=True)
    f.add_argument("--kernel", required=True)
    f.add_argument("--title", required=True)
    f.add_argument("--command", required=True)
    f.add_argument("--algorithmic-bytes", type=int, default=0)
    f.add_argument("--algorithmic-note", default="")
    f.add_argument("--out", required=True)
    c = sub.add_parser("counters")
    c.add_argument("files", nargs="+")
    c.add_argument("--title", required=True)
    c.add_argument("--command", action="append", required=True)
    c.add_argument("--note", default="")
    c.add_argument("--keep-copies", action="store_true", help="keep the runtime's copy / fill kernels in the table")
    c.add_argument("--out", required=True)
    a = ap.parse_args()
    if a.cmd == "trace":
        trace(a)
    elif a.cmd == "traffic":
        traffic(a)
    else:
        counters(a)


if __name__ == "__main__":
    main()
