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
    a = ap.parse_args()
    if a.cmd == "trace":
        trace(a)
    else:
        traffic(a)


if __name__ == "__main__":
    main()
